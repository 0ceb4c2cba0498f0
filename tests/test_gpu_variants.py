"""GPU parity for the appendix variants (gate functions, partial-mask ablations, Top-K routing) and
the output projection / whole FFN, through the C ABI, against the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import mglu_oracle as oracle
from paper_2506_23225_amd import api, synth
from tests.helpers import TOL, rel_err, to_np64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# token counts that land on the resident, panel and tiled kernels
KERNEL_TOKENS = [1, 5, 32, 100]


def _packed(x, W, masks):
    T, h = x.shape
    d, n_m = W.shape[1], masks.shape[0]
    desc = api.make_desc(T, h, d, n_m, x.dtype)
    return desc, api.mglu_pack_weights(desc, W), api.mglu_pack_masks(desc, masks)


@pytest.mark.parametrize("T", KERNEL_TOKENS)
@pytest.mark.parametrize("gate", ["gelu", "relu"])
def test_gate_functions(T, gate):
    x, W, masks = synth.make_inputs(640, 176, 4, T, dtype="bf16", seed=T, device=DEV)
    desc, Wp, Mp = _packed(x, W, masks)
    out = api.mglu_forward_variant(desc, x, Wp, Mp, gate=gate)
    ref = oracle.mglu_forward_variant(to_np64(x), to_np64(W), masks.cpu().numpy(), gate=gate)
    assert rel_err(to_np64(out), ref) <= TOL[x.dtype]


@pytest.mark.parametrize("T", KERNEL_TOKENS)
@pytest.mark.parametrize("mask_use", ["dense_gate", "dense_value", "none"])
def test_partial_mask_ablations(T, mask_use):
    x, W, masks = synth.make_inputs(512, 144, 2, T, dtype="bf16", seed=10 + T, device=DEV)
    desc, Wp, Mp = _packed(x, W, masks)
    out = api.mglu_forward_variant(desc, x, Wp, Mp, mask_use=mask_use)
    ref = oracle.mglu_forward_variant(to_np64(x), to_np64(W), masks.cpu().numpy(), mask_use=mask_use)
    assert rel_err(to_np64(out), ref) <= TOL[x.dtype]


def test_variants_fp32():
    x, W, masks = synth.make_inputs(256, 96, 3, 6, dtype="f32", seed=3, device=DEV)
    desc, Wp, Mp = _packed(x, W, masks)
    out = api.mglu_forward_variant(desc, x, Wp, Mp, gate="gelu", mask_use="dense_value")
    ref = oracle.mglu_forward_variant(to_np64(x), to_np64(W), masks.cpu().numpy(), gate="gelu", mask_use="dense_value")
    assert rel_err(to_np64(out), ref) <= TOL[x.dtype]


@pytest.mark.parametrize("dtype", ["bf16", "f32", "f16"])
@pytest.mark.parametrize("T,k", [(1, 2), (16, 1), (300, 3), (64, 8)])
def test_router_topk(dtype, T, k):
    h, n_m = 384, 8
    x, _, _ = synth.make_inputs(h, 16, 1, T, dtype=dtype, seed=T + k, device=DEV)
    gen = torch.Generator(device=DEV).manual_seed(99)
    Wr = (torch.randn(h, n_m, generator=gen, device=DEV) * 0.1).to(x.dtype)
    desc = api.make_desc(T, h, 16, n_m, x.dtype)
    w = api.mglu_route_topk(desc, x, Wr, k)
    ref = oracle.route_topk(to_np64(x), to_np64(Wr), k)
    got = to_np64(w)
    # the kept set is decided by floating point: compare tokens whose k-th and (k+1)-th logits are
    # clearly apart; for the rest only check that the result is a valid routing
    logits = np.sort(to_np64(x) @ to_np64(Wr), axis=1)[:, ::-1]
    clear = np.ones(T, bool) if k == n_m else (logits[:, k - 1] - logits[:, k]) > 1e-3
    assert clear.mean() > 0.9
    assert np.max(np.abs(got[clear] - ref[clear])) <= 1e-5
    assert np.all((got > 0).sum(axis=1) == k)
    np.testing.assert_allclose(got.sum(axis=1), 1.0, rtol=1e-5)


@pytest.mark.parametrize("T", [1, 4, 16, 33, 130])
def test_routed_layer_with_inactive_masks(T):
    """Top-2 of 8: the weights come from the GPU router and are handed to the oracle as they are, so
    only the routed layer itself is compared.  For T <= 16 unselected masks are skipped in the kernel."""
    h, d, n_m = 768, 208, 8
    x, W, masks = synth.make_inputs(h, d, n_m, T, dtype="bf16", seed=20 + T, device=DEV)
    gen = torch.Generator(device=DEV).manual_seed(5)
    Wr = (torch.randn(h, n_m, generator=gen, device=DEV) * 0.1).to(x.dtype)
    desc, Wp, Mp = _packed(x, W, masks)
    w = api.mglu_route_topk(desc, x, Wr, 2)
    out = api.mglu_forward_variant(desc, x, Wp, Mp, route_weights=w)
    ref = oracle.mglu_forward_variant(to_np64(x), to_np64(W), masks.cpu().numpy(), route=to_np64(w))
    assert rel_err(to_np64(out), ref) <= TOL[x.dtype]
    # all-ones weights reproduce the unrouted layer bit for bit
    ones = torch.ones(T, n_m, dtype=torch.float32, device=DEV)
    assert torch.equal(api.mglu_forward_variant(desc, x, Wp, Mp, route_weights=ones), api.mglu_forward(desc, x, Wp, Mp))


@pytest.mark.parametrize("dtype", ["bf16", "f32", "f16"])
def test_routed_layer_hand_made_weights(dtype):
    """Weights written by hand: one mask only, masks that differ from token to token, a token with no
    mask at all (its output is exactly 0), and no mask for any token (the whole output is exactly 0)."""
    h, d, n_m, T = 640, 112, 8, 3
    x, W, masks = synth.make_inputs(h, d, n_m, T, dtype=dtype, seed=77, device=DEV)
    desc, Wp, Mp = _packed(x, W, masks)
    w = torch.zeros(T, n_m, dtype=torch.float32, device=DEV)
    w[0, 5] = 1.0
    w[1, 0], w[1, 7] = 0.25, 0.75
    out = api.mglu_forward_variant(desc, x, Wp, Mp, route_weights=w)
    ref = oracle.mglu_forward_variant(to_np64(x), to_np64(W), masks.cpu().numpy(), route=to_np64(w))
    assert rel_err(to_np64(out), ref) <= TOL[x.dtype]
    assert torch.count_nonzero(out[2]) == 0
    out0 = api.mglu_forward_variant(desc, x, Wp, Mp, route_weights=torch.zeros_like(w))
    assert torch.count_nonzero(out0) == 0
    # one token, one mask: the n_m = 1 layer of that mask
    d1 = api.make_desc(1, h, d, 1, x.dtype)
    single = api.mglu_forward(d1, x[:1].contiguous(), Wp, api.mglu_pack_masks(d1, masks[5:6].contiguous()))
    assert torch.equal(api.mglu_forward_variant(api.make_desc(1, h, d, n_m, x.dtype), x[:1].contiguous(), Wp, Mp,
                                                route_weights=w[:1].contiguous()), single)


@pytest.mark.parametrize("T", [1, 8, 48, 100])
def test_sixteen_masks_routed_top4_gelu(T):
    """16 masks, top-4 routing from the GPU router, GELU gate: router, compaction and epilogue at the widest."""
    h, d, n_m = 512, 96, 16
    x, W, masks = synth.make_inputs(h, d, n_m, T, dtype="bf16", seed=300 + T, device=DEV)
    gen = torch.Generator(device=DEV).manual_seed(7)
    Wr = (torch.randn(h, n_m, generator=gen, device=DEV) * 0.1).to(x.dtype)
    desc, Wp, Mp = _packed(x, W, masks)
    w = api.mglu_route_topk(desc, x, Wr, 4)
    assert torch.all((w > 0).sum(dim=1) == 4)
    out = api.mglu_forward_variant(desc, x, Wp, Mp, gate="gelu", route_weights=w)
    ref = oracle.mglu_forward_variant(to_np64(x), to_np64(W), masks.cpu().numpy(), gate="gelu", route=to_np64(w))
    assert rel_err(to_np64(out), ref) <= TOL[x.dtype]


def test_variant_four_masks_tall_tile():
    """A launch large enough for the 128-token tile of the four-mask tiled kernel, in the variant mode:
    top-2 routing of 4 masks with a GELU gate, ragged tails."""
    h, d, n_m, T = 264, 4000, 4, 1000
    x, W, masks = synth.make_inputs(h, d, n_m, T, dtype="bf16", seed=41, device=DEV)
    gen = torch.Generator(device=DEV).manual_seed(9)
    Wr = (torch.randn(h, n_m, generator=gen, device=DEV) * 0.1).to(x.dtype)
    desc, Wp, Mp = _packed(x, W, masks)
    w = api.mglu_route_topk(desc, x, Wr, 2)
    out = api.mglu_forward_variant(desc, x, Wp, Mp, gate="gelu", route_weights=w)
    ref = oracle.mglu_forward_variant(to_np64(x), to_np64(W), masks.cpu().numpy(), gate="gelu", route=to_np64(w))
    assert rel_err(to_np64(out), ref) <= TOL[x.dtype]
    ones = torch.ones(T, n_m, dtype=torch.float32, device=DEV)
    assert torch.equal(api.mglu_forward_variant(desc, x, Wp, Mp, route_weights=ones), api.mglu_forward(desc, x, Wp, Mp))


@pytest.mark.parametrize("dtype,T", [("bf16", 1), ("bf16", 32), ("bf16", 200), ("f32", 3), ("f16", 5), ("f16", 120)])
def test_linear_projection(dtype, T):
    K, N = 656, 272
    a, W, _ = synth.make_inputs(K, N, 1, T, dtype=dtype, seed=T, device=DEV)
    desc = api.make_desc(T, K, N, 1, a.dtype)
    out = api.mglu_linear_forward(desc, a, api.mglu_pack_weights(desc, W))
    ref = oracle.linear_forward(to_np64(a), to_np64(W))
    assert rel_err(to_np64(out), ref) <= TOL[a.dtype]


def test_linear_projection_wide_tile():
    """A projection large enough for the tiled kernel's 512-column tile (the small ones above take the
    256-column tile), with ragged token, column and reduction tails."""
    T, K, N = 2100, 264, 4000
    a, W, _ = synth.make_inputs(K, N, 1, T, dtype="bf16", seed=5, device=DEV)
    desc = api.make_desc(T, K, N, 1, a.dtype)
    out = api.mglu_linear_forward(desc, a, api.mglu_pack_weights(desc, W))
    ref = oracle.linear_forward(to_np64(a), to_np64(W))
    assert rel_err(to_np64(out), ref) <= TOL[a.dtype]


@pytest.mark.parametrize("T,n_m", [(1, 4), (16, 4), (96, 4), (40, 12)])
def test_whole_ffn_block(T, n_m):
    """y = MGLU(x) Wo.  The GPU rounds the intermediate representation to bf16 between the two
    launches; the oracle does not, which is inside the bf16 tolerance.  (40 tokens, 12 masks: the layer
    itself is two launches with a hand-over through the workspace.)"""
    h, d = 512, 1408
    x, W, masks = synth.make_inputs(h, d, n_m, T, dtype="bf16", seed=T, device=DEV)
    gen = torch.Generator(device=DEV).manual_seed(11)
    Wo = (torch.randn(d, h, generator=gen, device=DEV) * 0.02).to(x.dtype)
    desc, Wp, Mp = _packed(x, W, masks)
    down = api.make_desc(T, d, h, 1, x.dtype)
    Wop = api.mglu_pack_weights(down, Wo)
    y, hidden = api.mglu_ffn_forward(desc, x, Wp, Mp, Wop)
    ref_hidden = oracle.mglu_forward(to_np64(x), to_np64(W), masks.cpu().numpy())
    ref = oracle.linear_forward(ref_hidden, to_np64(Wo))
    assert rel_err(to_np64(hidden), ref_hidden) <= TOL[x.dtype]
    assert rel_err(to_np64(y), ref) <= TOL[x.dtype]
