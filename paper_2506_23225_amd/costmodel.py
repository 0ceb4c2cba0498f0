"""Algorithmic bytes and FLOPs of one MGLU projection, for roofline reporting.

Memory-load model of the paper's Table "Parameter count and memory-access cost
per token": a linear unit loads 16*h*d bits, a GLU 32*h*d, an MGLU
(16 + n_m)*h*d (16-bit weights, one bit per mask per weight element).
Compute: one dense contraction for the unmasked sum plus one per mask, the
value branches coming from the complement for free.
"""

WEIGHT_BITS = {"bf16": 16, "f32": 32, "f16": 16}


def mglu_weight_bits(d_model, d_ff, n_masks, dtype="bf16"):
    """Bits of W plus its n_masks bit planes: (16 + n_m) h d for 16-bit weights."""
    return (WEIGHT_BITS[dtype] + n_masks) * d_model * d_ff


def glu_weight_bits(d_model, d_ff, dtype="bf16"):
    """Bits of the two GLU matrices: 32 h d for 16-bit weights."""
    return 2 * WEIGHT_BITS[dtype] * d_model * d_ff


def mglu_bytes(d_model, d_ff, n_masks, tokens, dtype="bf16"):
    """Bytes one call must move: W, masks, x in and out out, each exactly once."""
    act = WEIGHT_BITS[dtype] // 8
    return (mglu_weight_bits(d_model, d_ff, n_masks, dtype) // 8
            + act * tokens * d_model + act * tokens * d_ff)


def glu_bytes(d_model, d_ff, tokens, dtype="bf16"):
    act = WEIGHT_BITS[dtype] // 8
    return glu_weight_bits(d_model, d_ff, dtype) // 8 + act * tokens * (d_model + d_ff)


def mglu_flops(d_model, d_ff, n_masks, tokens):
    """2 T h d (1 + n_m): the unmasked contraction plus one masked contraction per mask."""
    return 2 * tokens * d_model * d_ff * (1 + n_masks)


def glu_flops(d_model, d_ff, tokens):
    return 4 * tokens * d_model * d_ff
