"""The packed layouts as documented (include/mglu.h calls them opaque; the kernels' header and the design
notes state them): pack on the GPU, copy the buffer back and decode it on the host with an independent
reading of the documented layout -- every weight and every mask bit must come back, and padding must be zero.

Layouts (column blocks jb of 16, reduction chunks kc of 128, lane l = 16 q + r):
  16-bit weights  [jb][kc][tile t<4][lane][e<8]   = W[128 kc + 32 t + 8 q + e][16 jb + r]
  fp32 weights    [jb][kc][tile t<8][lane][e<4]   = W[128 kc + 16 t + 4 q + e][16 jb + r]
  masks           NMP = n_masks rounded up to 1, 2, 4, 8, 16 words per lane and chunk:
                  [jb][kc][lane][word<NMP], or for NMP >= 8 [jb][kc][piece<NMP/4][lane][word<4]
    16-bit: element (t, e) -> pair p = e / 2, half hf = e % 2, bit position + 16 hf in word
            NMP 1: word 0, bit 4t + p;  2: word p/2, bit 2(2t + p%2) + i;  4: word 2(t/2) + p/2, bit 4(2(t%2) + p%2) + i;
            8: word 2t + p/2, bit 8(p%2) + i;  16: word 8(i/8) + 2t + p/2, bit 8(p%2) + i%8
    fp32:   element E = 4t + e, linear = E NMP + i -> word linear / 32, bit linear % 32
  planar masks    [jb][mask i][kc][lane], bit 4t + e/2 + 16(e%2) (16-bit) or 4t + e (fp32)
"""
import numpy as np
import pytest
import torch

from paper_2506_23225_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _geometry(h, d, fp32):
    NB, NC = -(-d // 16), -(-h // 128)
    tiles, per = (8, 4) if fp32 else (4, 8)
    jb, kc, t, lane, e = np.meshgrid(np.arange(NB), np.arange(NC), np.arange(tiles), np.arange(64), np.arange(per),
                                     indexing="ij")
    k = 128 * kc + (128 // tiles) * t + per * (lane // 16) + e
    j = 16 * jb + lane % 16
    return NB, NC, tiles, per, jb, kc, t, lane, e, k, j


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("layout", ["kn", "nk"])
def test_packed_weights_layout(dtype, layout):
    h, d = 264, 40
    _, W, _ = synth.make_inputs(h, d, 1, 1, dtype=dtype, seed=3, device=DEV)
    desc = api.make_desc(1, h, d, 1, W.dtype, layout)
    src = W.t().contiguous() if layout == "nk" else W
    packed = api.mglu_pack_weights(desc, src)
    NB, NC, tiles, per, jb, kc, t, lane, e, k, j = _geometry(h, d, dtype == "f32")
    got = packed.view(W.dtype).cpu().to(torch.float64).numpy().reshape(NB, NC, tiles, 64, per)
    Wn = np.zeros((NC * 128, NB * 16))
    Wn[:h, :d] = W.cpu().to(torch.float64).numpy()
    assert np.array_equal(got, Wn[k, j])      # exact: packing moves bits, padding is zero


def _mask_word_bit(nmp, fp32, t, e, i):
    if fp32:
        lin = (4 * t + e) * nmp + i
        return lin // 32, lin % 32
    p, hf = e // 2, e % 2
    if nmp == 1:
        w, b = 0, 4 * t + p
    elif nmp == 2:
        w, b = p // 2, 2 * (2 * t + p % 2) + i
    elif nmp == 4:
        w, b = 2 * (t // 2) + p // 2, 4 * (2 * (t % 2) + p % 2) + i
    elif nmp == 8:
        w, b = 2 * t + p // 2, 8 * (p % 2) + i
    else:
        w, b = 8 * (i // 8) + 2 * t + p // 2, 8 * (p % 2) + i % 8
    return w, b + 16 * hf


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("n_m", [1, 2, 3, 4, 7, 8, 11, 16])
def test_packed_masks_layout(dtype, n_m):
    h, d = 264, 40
    _, W, masks = synth.make_inputs(h, d, n_m, 1, dtype=dtype, seed=n_m, device=DEV)
    desc = api.make_desc(1, h, d, n_m, W.dtype)
    nmp = next(v for v in (1, 2, 4, 8, 16) if v >= n_m)
    assert api.mglu_packed_mask_bytes(desc) == -(-d // 16) * -(-h // 128) * 64 * nmp * 4
    words = api.mglu_pack_masks(desc, masks).cpu().numpy().view(np.uint32)
    fp32 = dtype == "f32"
    NB, NC, tiles, per, jb, kc, t, lane, e, k, j = _geometry(h, d, fp32)
    if nmp >= 8:
        words = words.reshape(NB, NC, nmp // 4, 64, 4).transpose(0, 1, 3, 2, 4).reshape(NB, NC, 64, nmp)
    else:
        words = words.reshape(NB, NC, 64, nmp)
    M = np.zeros((nmp, NC * 128, NB * 16), dtype=np.uint32)
    M[:n_m, :h, :d] = masks.cpu().numpy()
    seen = np.zeros_like(words)
    for i in range(nmp):
        w, b = _mask_word_bit(nmp, fp32, t, e, i)
        bits = (words[jb, kc, lane, w] >> b.astype(np.uint32)) & 1
        assert np.array_equal(bits, M[i][k, j]), "mask %d" % i
        np.bitwise_or.at(seen, (jb, kc, lane, w), np.uint32(1) << b.astype(np.uint32))
    assert np.all(seen == 0xFFFFFFFF)         # the positions above cover every bit of every word exactly


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("n_m", [1, 3, 8, 16])
def test_planar_masks_layout(dtype, n_m):
    h, d = 264, 40
    _, W, masks = synth.make_inputs(h, d, n_m, 1, dtype=dtype, seed=20 + n_m, device=DEV)
    desc = api.make_desc(1, h, d, n_m, W.dtype)
    fp32 = dtype == "f32"
    NB, NC, tiles, per, jb, kc, t, lane, e, k, j = _geometry(h, d, fp32)
    assert api.mglu_packed_mask_bytes_planar(desc) == NB * NC * 64 * n_m * 4
    words = api.mglu_pack_masks_planar(desc, masks).cpu().numpy().view(np.uint32).reshape(NB, n_m, NC, 64)
    M = np.zeros((n_m, NC * 128, NB * 16), dtype=np.uint32)
    M[:, :h, :d] = masks.cpu().numpy()
    bit = (4 * t + e) if fp32 else (4 * t + e // 2 + 16 * (e % 2))
    for i in range(n_m):
        assert np.array_equal((words[jb, i, kc, lane] >> bit.astype(np.uint32)) & 1, M[i][k, j]), "mask %d" % i
