"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by element."""
import numpy as np
import pytest
import torch

from oracle import mglu_oracle as oracle
from paper_2506_23225_amd import api, synth
from tests.helpers import TOL, edge_columns, rel_err, to_np64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(x, W, masks, layout="kn", via_bool=False):
    T, h = x.shape
    n_m = masks.shape[0]
    d = W.shape[1] if layout == "kn" else W.shape[0]
    desc = api.make_desc(T, h, d, n_m, x.dtype, layout)
    if via_bool:
        return api.mglu_forward_bool(desc, x, W, masks)
    Wp = api.mglu_pack_weights(desc, W)
    Mp = api.mglu_pack_masks(desc, masks)
    return api.mglu_forward(desc, x, Wp, Mp)


def _check_full(x, W, masks, out, tol=None):
    ref = oracle.mglu_forward(to_np64(x), to_np64(W), masks.cpu().numpy())
    err = rel_err(to_np64(out), ref)
    assert err <= (tol or TOL[x.dtype]), err
    return err


def _check_columns(x, W, masks, out, cols):
    ci = torch.as_tensor(cols, device=W.device)
    ref = oracle.mglu_forward(to_np64(x), to_np64(W[:, ci]), masks[:, :, ci].cpu().numpy())
    err = rel_err(to_np64(out[:, ci]), ref)
    assert err <= TOL[x.dtype], err
    return err


def test_tiny_fp32_config():
    cfg = synth.config("tiny")
    x, W, masks = synth.make_inputs(**cfg, seed=0, device=DEV)
    out = _run(x, W, masks)
    print("tiny fp32 rel err", _check_full(x, W, masks, out))


@pytest.mark.parametrize("dtype", ["bf16", "f32", "f16"])
@pytest.mark.parametrize("T,h,d,n_m", [
    (1, 8, 1, 1), (1, 128, 16, 1), (3, 200, 50, 3), (16, 256, 688, 2), (17, 136, 17, 5),
    (33, 1024, 100, 8), (5, 2048, 48, 4), (2, 520, 36, 7), (64, 384, 64, 1), (70, 256, 40, 2),
])
def test_ragged_shapes(dtype, T, h, d, n_m):
    x, W, masks = synth.make_inputs(h, d, n_m, T, dtype=dtype, seed=T + h + d, device=DEV)
    _check_full(x, W, masks, _run(x, W, masks))


@pytest.mark.parametrize("T,h,d,n_m", [(40, 384, 25616, 2), (17, 136, 25608, 8), (64, 640, 25600, 1)])
def test_wide_panel_shape_ragged(T, h, d, n_m):
    """d_ff large enough for the 8-column-block workgroup shape of the panel kernel, with a ragged
    column tail, an odd number of K chunks and token counts that leave partial token blocks."""
    x, W, masks = synth.make_inputs(h, d, n_m, T, dtype="bf16", seed=T + h + d, device=DEV)
    out = _run(x, W, masks)
    cols = edge_columns(d, n_random=256, seed=T)
    _check_columns(x, W, masks, out, cols)


@pytest.mark.parametrize("T,h,d,n_m", [
    (65, 128, 16, 1), (128, 256, 128, 4), (200, 520, 272, 4), (300, 384, 1000, 8), (129, 1024, 130, 2),
    (257, 136, 2064, 1), (1100, 256, 300, 3), (96, 2048, 144, 8),
])
def test_prefill_kernel_ragged_shapes(T, h, d, n_m):
    """Token counts beyond one pass of the streaming kernels take the MFMA-tiled kernel: ragged token, column and
    reduction tails."""
    x, W, masks = synth.make_inputs(h, d, n_m, T, dtype="bf16", seed=T + h + d, device=DEV)
    _check_full(x, W, masks, _run(x, W, masks))


@pytest.mark.parametrize("dtype,T,h,d,n_m", [
    ("bf16", 1000, 320, 4000, 4), ("bf16", 1000, 136, 4090, 3), ("f16", 1000, 264, 4000, 4), ("bf16", 250, 256, 16300, 4),
])
def test_prefill_four_masks_tall_tile(dtype, T, h, d, n_m):
    """With three or four masks the tiled kernel picks one of four tile shapes per launch (whichever covers
    the chip in the least estimated time).  These launches are large enough for the 8-wavefront 128-token
    tile, with ragged token, column and reduction tails; the other three shapes have cases of their own
    below and in tests/test_gpu_plan_parity.py."""
    x, W, masks = synth.make_inputs(h, d, n_m, T, dtype=dtype, seed=T + h + d, device=DEV)
    out = _run(x, W, masks)
    if d > 4096:
        _check_columns(x, W, masks, out, edge_columns(d, n_random=256, seed=T))
    else:
        _check_full(x, W, masks, out)


@pytest.mark.parametrize("dtype,T,h,d,n_m,tile", [
    ("bf16", 80, 264, 28672, 4, "1, 6, 0, 2, 8"), ("bf16", 96, 136, 28660, 3, "1, 6, 0, 2, 8"),
    ("f16", 70, 392, 28672, 4, "1, 6, 0, 2, 8"), ("bf16", 390, 264, 28672, 4, "1, 8, 0, 3, 4"),
    ("bf16", 400, 136, 28650, 3, "1, 8, 0, 3, 4"), ("bf16", 100, 520, 1000, 4, "1, 4, 0, 6, 4"),
])
def test_prefill_four_masks_other_tiles(dtype, T, h, d, n_m, tile):
    """The four-mask kernel's 96-token mask-major tile, its 4-wavefront 128-token tile and its 4-wavefront
    64-token tile, each asserted through the plan query, on ragged shapes."""
    x, W, masks = synth.make_inputs(h, d, n_m, T, dtype=dtype, seed=T + h + d, device=DEV)
    traits = {"bf16": "Bf16Traits", "f16": "F16Traits"}[dtype]
    assert api.mglu_describe_plan(api.make_desc(T, h, d, n_m, x.dtype)) == "prefill_kernel<%s, 4, %s>" % (traits, tile)
    out = _run(x, W, masks)
    if d > 4096:
        _check_columns(x, W, masks, out, edge_columns(d, n_random=128, seed=T))
    else:
        _check_full(x, W, masks, out)


def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(n):
        n_m = int(rng.choice([1, 2, 3, 4, 5, 8, 11, 16]))
        T = int(rng.choice([rng.integers(1, 17), rng.integers(17, 65), rng.integers(65, 300)]))
        h = 8 * int(rng.integers(2, 81))          # 16 .. 640, any multiple of 8
        d = int(rng.integers(1, 600))
        shapes.append((str(rng.choice(["bf16", "f16"])), T, h, d, n_m))
    return shapes


@pytest.mark.parametrize("dtype,T,h,d,n_m", _random_shapes(40, seed=2506))
def test_random_shapes(dtype, T, h, d, n_m):
    """Seeded random shapes across the hand-over points between the kernels and their tile shapes: any token
    count up to 300, any d_model that is a multiple of 8, any d_ff, the mask counts of every instantiation."""
    x, W, masks = synth.make_inputs(h, d, n_m, T, dtype=dtype, seed=T + h + d + n_m, device=DEV)
    _check_full(x, W, masks, _run(x, W, masks))


@pytest.mark.parametrize("T,h,d,n_m", [(40, 384, 25616, 2), (200, 520, 272, 4), (300, 384, 1000, 8), (129, 1024, 130, 1)])
def test_fp16_panel_and_tiled_kernels(T, h, d, n_m):
    """fp16, the paper's own precision, through the panel kernel and the MFMA-tiled kernel."""
    x, W, masks = synth.make_inputs(h, d, n_m, T, dtype="f16", seed=T + h + d, device=DEV)
    out = _run(x, W, masks)
    if d > 4096:
        _check_columns(x, W, masks, out, edge_columns(d, n_random=256, seed=T))
    else:
        _check_full(x, W, masks, out)


@pytest.mark.parametrize("dtype,T,h,d,n_m", [
    ("bf16", 1, 2048, 176, 16), ("bf16", 3, 520, 100, 9), ("bf16", 16, 384, 64, 12), ("bf16", 40, 640, 272, 16),
    ("bf16", 64, 256, 25616, 16), ("bf16", 130, 520, 200, 13), ("bf16", 300, 1024, 144, 16), ("f16", 2, 1024, 80, 16),
    ("f16", 200, 384, 136, 16), ("f32", 5, 264, 40, 16), ("f32", 33, 200, 24, 11),
    ("bf16", 70, 392, 101, 10), ("f16", 129, 264, 50, 9),
])
def test_nine_to_sixteen_masks(dtype, T, h, d, n_m):
    """More than 8 masks (the paper's largest ablation has 16): 17 accumulator sets and mask words in four
    pieces per chunk in the resident and panel kernels; above 16 tokens the tiled kernel runs once per
    8-mask half of the format with an fp32 hand-over (also with d_ff not a multiple of 4)."""
    x, W, masks = synth.make_inputs(h, d, n_m, T, dtype=dtype, seed=T + h + n_m, device=DEV)
    out = _run(x, W, masks)
    if d > 4096:
        _check_columns(x, W, masks, out, edge_columns(d, n_random=128, seed=T))
    else:
        _check_full(x, W, masks, out)


@pytest.mark.parametrize("T", [1, 4096])
def test_fp16_paper_shape_sampled(T):
    """4096 x 14336 with 4 masks in fp16: the shape and precision of the paper's kernel timings."""
    cfg = synth.config("prefill_8b", tokens=T, dtype="f16")
    x, W, masks = synth.make_inputs(**cfg, seed=0, device=DEV)
    out = _run(x, W, masks)
    print("fp16 4096x14336 T=%d rel err" % T,
          _check_columns(x, W, masks, out, edge_columns(cfg["d_ff"], n_random=48 if T > 1 else 128)))


@pytest.mark.parametrize("n_m,T", [(2, 64), (6, 32), (12, 16)])
def test_kernel_hand_over(n_m, T):
    """T tokens -- what the streaming (panel) kernel covers in one pass over W with this many masks -- run
    on it, T + 1 on the MFMA-tiled one: both against the oracle, and the shared rows against each other
    (they may differ by summation order only)."""
    x, W, masks = synth.make_inputs(768, 272, n_m, T + 1, dtype="bf16", seed=64 + n_m, device=DEV)
    more = _run(x, W, masks)
    fewer = _run(x[:T].contiguous(), W, masks)
    _check_full(x, W, masks, more)
    _check_full(x[:T], W, masks, fewer)
    assert rel_err(to_np64(fewer), to_np64(more[:T])) <= 1e-2


def test_prefill_kernel_other_layout_and_entries():
    """The tiled kernel through the NK layout, the unpacked-input entry and non-0/1 mask bytes."""
    x, W, masks = synth.make_inputs(520, 200, 7, 130, dtype="bf16", seed=9, device=DEV)
    ref = _run(x, W, masks)
    _check_full(x, W, masks, ref)
    Wt, Mt = W.t().contiguous(), masks.transpose(1, 2).contiguous()
    assert torch.equal(_run(x, Wt, Mt, layout="nk"), ref)
    assert torch.equal(_run(x, W, masks, via_bool=True), ref)
    assert torch.equal(_run(x, W, masks * 255), ref)           # any non-zero byte means "gate"


@pytest.mark.parametrize("dtype", ["bf16", "f32", "f16"])
def test_nk_layout_and_bool_entry(dtype):
    x, W, masks = synth.make_inputs(392, 72, 3, 4, dtype=dtype, seed=5, device=DEV)
    ref = _run(x, W, masks)
    Wt = W.t().contiguous()
    Mt = masks.transpose(1, 2).contiguous()
    assert torch.equal(_run(x, Wt, Mt, layout="nk"), ref)
    assert torch.equal(_run(x, W, masks, via_bool=True), ref)
    assert torch.equal(_run(x, Wt, Mt, layout="nk", via_bool=True), ref)
    _check_full(x, W, masks, ref)


def test_decode_gemv_config_full():
    cfg = synth.config("decode_gemv")
    x, W, masks = synth.make_inputs(**cfg, seed=0, device=DEV)
    out = _run(x, W, masks)
    print("decode_gemv rel err", _check_full(x, W, masks, out))


@pytest.mark.parametrize("T", [1, 4, 16])
def test_decode_8b_config_sampled(T):
    cfg = synth.config("decode_8b", tokens=T)
    x, W, masks = synth.make_inputs(**cfg, seed=0, device=DEV)
    out = _run(x, W, masks)
    print("decode_8b T=%d rel err" % T, _check_columns(x, W, masks, out, edge_columns(cfg["d_ff"])))


def test_decode_8b_sixteen_masks_sampled():
    """4096 x 14336 with 16 masks at one token: the benchmark's 16-mask decode row."""
    cfg = synth.config("decode_8b", n_masks=16, tokens=1)
    x, W, masks = synth.make_inputs(**cfg, seed=0, device=DEV)
    assert api.mglu_describe_plan(api.make_desc(1, 4096, 14336, 16, x.dtype)) == \
        "stream_resident_kernel<Bf16Traits, 16, 0, 2, false>"
    out = _run(x, W, masks)
    print("decode_8b n_m=16 rel err", _check_columns(x, W, masks, out, edge_columns(cfg["d_ff"])))


def test_prefill_8b_sixteen_masks_sampled():
    """4096 x 14336 with 16 masks at 4096 tokens, the benchmark's 16-mask prefill row: two launches of the
    8-mask tiled kernel with the fp32 hand-over, all tokens on sampled columns."""
    cfg = synth.config("prefill_8b", n_masks=16)
    x, W, masks = synth.make_inputs(**cfg, seed=0, device=DEV)
    assert api.mglu_describe_plan(api.make_desc(cfg["tokens"], 4096, 14336, 16, x.dtype)) == \
        "prefill_kernel<Bf16Traits, 8, 1, 4, 0, 2, 8> twice"
    out = _run(x, W, masks)
    print("prefill_8b n_m=16 rel err", _check_columns(x, W, masks, out, edge_columns(cfg["d_ff"], n_random=8)))


def test_prefill_8b_config_sampled():
    """Full-size prefill configuration: all 4096 tokens on sampled columns (tile edges, tail, random)."""
    cfg = synth.config("prefill_8b")
    x, W, masks = synth.make_inputs(**cfg, seed=0, device=DEV)
    out = _run(x, W, masks)
    print("prefill_8b rel err", _check_columns(x, W, masks, out, edge_columns(cfg["d_ff"], n_random=48)))


@pytest.mark.parametrize("T", [1, 32, 2048])
@pytest.mark.parametrize("n_m", [1, 2, 4, 8])
def test_large_config_sampled(n_m, T):
    """Every cell of the large layer sweep (8192 x 28672), each in the launch configuration the benchmark times."""
    cfg = synth.config("large", n_masks=n_m, tokens=T)
    x, W, masks = synth.make_inputs(**cfg, seed=0, device=DEV)
    out = _run(x, W, masks)
    print("large n_m=%d T=%d rel err" % (n_m, T),
          _check_columns(x, W, masks, out, edge_columns(cfg["d_ff"], n_random=64)))


def test_projections_partition_and_oracle():
    """Alg. 1's z: gate_i + value_i = xW, and each branch matches the oracle's."""
    x, W, masks = synth.make_inputs(512, 96, 4, 3, dtype="bf16", seed=11, device=DEV)
    desc = api.make_desc(3, 512, 96, 4, x.dtype)
    Wp, Mp = api.mglu_pack_weights(desc, W), api.mglu_pack_masks(desc, masks)
    t, gate, value = api.mglu_projections(desc, x, Wp, Mp)
    _, og, ov = oracle.mglu_forward(to_np64(x), to_np64(W), masks.cpu().numpy(), return_projections=True)
    dense = to_np64(x) @ to_np64(W)
    scale = np.abs(dense).max()
    assert np.abs(to_np64(t) - dense).max() <= 1e-5 * scale
    for i in range(4):
        assert np.abs(to_np64(gate[i]) - og[i]).max() <= 1e-5 * scale
        assert np.abs(to_np64(value[i]) - ov[i]).max() <= 1e-5 * scale
        assert np.abs(to_np64(gate[i] + value[i]) - dense).max() <= 1e-5 * scale


@pytest.mark.parametrize("dtype", ["bf16", "f32", "f16"])
def test_degenerate_masks_and_inputs(dtype):
    """Cases whose exact answer is 0.  All-value masks and one-hot inputs give 0 bit for bit.
    An all-gate mask gives value_i = (t + dsum_i)/2 with dsum_i the sum of the negated terms;
    the matrix cores' accumulation is not sign-symmetric to the last bit, so that case is held
    to an absolute bound far below one output ulp instead: 1e-6 * |x|_2 * max|W| * sqrt(h)."""
    h = 640
    x, W, masks = synth.make_inputs(h, 80, 2, 2, dtype=dtype, seed=3, device=DEV)
    ones = torch.ones_like(masks)
    bound = 1e-6 * float(x.float().norm(dim=1).max()) * float(W.float().abs().max()) * h ** 0.5
    assert float(_run(x, W, ones).float().abs().max()) <= bound   # all-gate: value branch empty
    assert torch.count_nonzero(_run(x, W, 1 - ones)) == 0          # all-value: swish(0) = 0
    xh = torch.zeros_like(x)
    xh[0, 77] = -3.25
    xh[1, 639] = 0.5
    assert torch.count_nonzero(_run(xh, W, masks)) == 0            # one-hot rows
    # an extra all-value route adds exactly nothing, an extra all-gate route at most the bound
    base = _run(x, W, masks)
    assert torch.equal(_run(x, W, torch.cat([masks, 1 - ones[:1]])), base)
    more = _run(x, W, torch.cat([masks, ones[:1]]))
    assert rel_err(to_np64(more), to_np64(base)) <= {"bf16": 1e-2, "f16": 2e-3, "f32": 1e-5}[dtype]


def test_rows_independent_and_mask_order_and_determinism():
    x, W, masks = synth.make_inputs(1024, 160, 4, 16, dtype="bf16", seed=4, device=DEV)
    full = _run(x, W, masks)
    assert torch.equal(_run(x, W, masks), full)                 # same bits on a second call
    for tau in (0, 7, 15):
        assert torch.equal(_run(x[tau:tau + 1].contiguous(), W, masks)[0], full[tau])
    perm = _run(x, W, masks[[2, 0, 3, 1]].contiguous())
    assert rel_err(to_np64(perm), to_np64(full)) <= 1e-2       # fp32 sum order differs, value does not


@pytest.mark.parametrize("dtype,T", [("bf16", 1), ("bf16", 16), ("f32", 3), ("bf16", 150), ("f16", 2), ("f16", 90)])
def test_swiglu_reference_kernel(dtype, T):
    xg, Wg, _ = synth.make_inputs(768, 208, 1, T, dtype=dtype, seed=6, device=DEV)
    _, Wv, _ = synth.make_inputs(768, 208, 1, T, dtype=dtype, seed=7, device=DEV)
    desc = api.make_desc(T, 768, 208, 1, xg.dtype)
    out = api.swiglu_forward(desc, xg, api.mglu_pack_weights(desc, Wg), api.mglu_pack_weights(desc, Wv))
    ref = oracle.swiglu_forward(to_np64(xg), to_np64(Wg), to_np64(Wv))
    assert rel_err(to_np64(out), ref) <= TOL[xg.dtype]


def test_single_mask_equals_swiglu_kernel_on_split_matrices():
    """Eq. 2 vs Eq. 1 on the GPU: MGLU_1(W, M) against the two-matrix kernel fed W*M and W*(1-M)."""
    x, W, masks = synth.make_inputs(512, 128, 1, 4, dtype="bf16", seed=8, device=DEV)
    desc = api.make_desc(4, 512, 128, 1, x.dtype)
    m = masks[0].to(W.dtype)
    sw = api.swiglu_forward(desc, x, api.mglu_pack_weights(desc, (W * m).contiguous()),
                            api.mglu_pack_weights(desc, (W * (1 - m)).contiguous()))
    assert rel_err(to_np64(_run(x, W, masks)), to_np64(sw)) <= 1e-2
