"""Seeded synthetic inputs for the MGLU forward pass.

This module serves both the GPU path and the CPU oracle and therefore holds
none of the method's arithmetic: it only draws x, W and the masks.

Recipe (one generator per call, seeded; draw order x, then W, then the mask
planes one by one):
  x      ~ N(0, 1)            [tokens, d_model]
  W      ~ N(0, w_std^2)      [d_model, d_ff]   (logical: reduction index first)
  masks  ~ Bernoulli(0.5)     [n_masks, d_model, d_ff], drawn as uniform < 0.5
x and W are drawn in fp32 and, for the bf16 configurations, rounded once to
bf16 (nearest-even); both sides of a parity test then start from those very
values.  The shapes follow the Llama-style FFN up-projections the paper's
latency section measures; its trained masks are close to half ones, which the
Bernoulli(0.5) planes stand in for.
"""
import torch

# name -> shape and statistics of one workload.  `tokens` may be overridden.
CONFIGS = {
    "tiny":        dict(d_model=256,  d_ff=688,   n_masks=1, tokens=4,    dtype="f32",  w_std=0.02),
    "decode_gemv": dict(d_model=2048, d_ff=5632,  n_masks=4, tokens=1,    dtype="bf16", w_std=0.02),
    "decode_8b":   dict(d_model=4096, d_ff=14336, n_masks=8, tokens=1,    dtype="bf16", w_std=0.02),
    "prefill_8b":  dict(d_model=4096, d_ff=14336, n_masks=4, tokens=4096, dtype="bf16", w_std=0.02),
    "large":       dict(d_model=8192, d_ff=28672, n_masks=4, tokens=1,    dtype="bf16", w_std=0.01),
}

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


def config(name, **overrides):
    """A copy of a named workload with some fields replaced (e.g. tokens=16)."""
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    cfg["name"] = name
    return cfg


def make_inputs(d_model, d_ff, n_masks, tokens, dtype="bf16", w_std=0.02,
                seed=0, device="cpu", **_ignored):
    """Draw (x, W, masks) on `device`.

    x [tokens, d_model] and W [d_model, d_ff] in `dtype`; masks
    [n_masks, d_model, d_ff] as uint8 bytes 0/1.
    """
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    tdt = TORCH_DTYPE[dtype]
    x = torch.randn(tokens, d_model, generator=gen, device=device, dtype=torch.float32).to(tdt)
    W = (torch.randn(d_model, d_ff, generator=gen, device=device, dtype=torch.float32) * w_std).to(tdt)
    masks = torch.empty(n_masks, d_model, d_ff, dtype=torch.uint8, device=device)
    for i in range(n_masks):
        masks[i] = torch.rand(d_model, d_ff, generator=gen, device=device) < 0.5
    return x, W, masks
