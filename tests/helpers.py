"""Shared pieces of the parity tests: the error metric and the sampled-column oracle call."""
import numpy as np
import torch

# spec tolerances: max relative error, bf16 inputs 2e-2, fp32 inputs 1e-4; fp16 (not among
# the benchmark spec's types) gets the bf16 bar scaled by the ratio of the two formats' rounding units,
# 2^-11 / 2^-8: the final rounding to the output type dominates the error of both
TOL = {torch.bfloat16: 2e-2, torch.float32: 1e-4, torch.float16: 2.5e-3}


def rel_err(y, ref):
    """max |y - ref| / max(|ref|, rms(ref)): elementwise relative error with the
    denominator floored at the output's rms, so that outputs that happen to fall
    next to zero (where any finite-precision result has unbounded relative error)
    are judged against the typical output magnitude."""
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert y.shape == ref.shape, (y.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    den = np.maximum(np.abs(ref), max(rms, 1e-300))
    return float(np.max(np.abs(y - ref) / den))


def to_np64(t):
    return t.detach().to("cpu", torch.float64).numpy()


def edge_columns(d_ff, n_random=128, seed=0):
    """Columns around every tile boundary that matters (16 ... 512) plus the tail and a random sample."""
    cols = {0, d_ff - 1}
    for tile in (16, 32, 64, 128, 256, 512):
        for b in range(tile, d_ff, max(tile, (d_ff // 6) // tile * tile)):
            cols.update((b - 1, b))
        last = (d_ff - 1) // tile * tile
        cols.update((last - 1, last))
    rng = np.random.default_rng(seed)
    cols.update(int(c) for c in rng.integers(0, d_ff, size=n_random))
    return np.array(sorted(c for c in cols if 0 <= c < d_ff), dtype=np.int64)
