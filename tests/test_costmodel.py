"""The byte/FLOP model used for roofline reporting, pinned to the paper's worked numbers."""
import os

from paper_2506_23225_amd import costmodel as cm


def _golden(golden_dir):
    vals = {}
    with open(os.path.join(golden_dir, "memory_model.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            vals[k] = float(v)
    return vals


def test_memory_load_table(golden_dir):
    g = _golden(golden_dir)
    h, d = int(g["llama1b_h"]), int(g["llama1b_d"])
    glu = cm.glu_weight_bits(h, d)
    assert glu == 32 * h * d
    for n_m in (1, 2, 4, 8):
        assert cm.mglu_weight_bits(h, d, n_m) == (16 + n_m) * h * d
    assert (glu - cm.mglu_weight_bits(h, d, 1)) / glu == g["relative_saving_nm1"]
    assert (glu - cm.mglu_weight_bits(h, d, 4)) / glu == g["relative_saving_nm4"]
    MiB = 8 * 2 ** 20
    one_matrix = cm.glu_weight_bits(h, d) // 2
    assert 3 * one_matrix / MiB == g["llama1b_three_matrices_MiB"]
    assert 2 * one_matrix / MiB == g["llama1b_two_matrices_MiB"]
    assert (cm.mglu_weight_bits(h, d, 1) - one_matrix) / MiB == g["llama1b_mask_plane_MiB"]


def test_bytes_and_flops_at_the_benchmark_shapes():
    # decode GEMV: 2048 x 5632, four masks, one token
    assert cm.mglu_bytes(2048, 5632, 4, 1) == 23068672 + 5767168 + 2 * 2048 + 2 * 5632
    assert cm.mglu_flops(4096, 14336, 4, 4096) == 2 * 4096 * 4096 * 14336 * 5
    assert cm.glu_flops(4096, 14336, 4096) == 4 * 4096 * 4096 * 14336
    assert cm.glu_bytes(2048, 5632, 1) == 4 * 2048 * 5632 + 2 * (2048 + 5632)
