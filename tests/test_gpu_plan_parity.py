"""One oracle-parity case per kernel instantiation the library can select.

tests/plans.py asks the library (mglu_describe_plan) which kernel each descriptor of a grid runs and
keeps the cheapest descriptor per instantiation; tests/test_plan_coverage.py shows that the grid
reaches every kernel compiled into libmglu.so.  Here each of those descriptors is run through the C ABI
and compared with the fp64 oracle, so no selectable code path is without a parity check.
"""
import numpy as np
import pytest
import torch

from oracle import mglu_oracle as oracle
from paper_2506_23225_amd import api, synth
from tests import plans
from tests.helpers import TOL, edge_columns, rel_err, to_np64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

PLANS = sorted(plans.enumerate_plans().items())
# what the variant call switches on, in turn over the instantiations (the oracle gets the same choice)
VARIATIONS = (dict(gate="gelu"), dict(gate="relu", mask_use="dense_gate"), dict(route=True),
              dict(mask_use="dense_value"))


def _route_weights(T, n_m, seed, k=2):
    """Top-k-style weights: k non-zero entries per token summing to 1 (all of them when n_m < k)."""
    rng = np.random.default_rng(seed)
    w = np.zeros((T, n_m), dtype=np.float32)
    for t in range(T):
        keep = rng.choice(n_m, size=min(k, n_m), replace=False)
        v = rng.random(len(keep)).astype(np.float32) + 0.25
        w[t, keep] = v / v.sum()
    return w


@pytest.mark.parametrize("index", range(len(PLANS)), ids=[name for name, _ in PLANS])
def test_every_selectable_instantiation(index):
    plan, (_, dname, call, n_m, T, h, d, k) = PLANS[index]
    print("plan case:", plan, dname, call, "n_m=%d T=%d h=%d d=%d k=%d" % (n_m, T, h, d, k), flush=True)
    x, W, masks = synth.make_inputs(h, d, n_m, T, dtype=dname, seed=index, device=DEV)
    desc = api.make_desc(T, h, d, n_m, x.dtype)
    assert api.mglu_describe_plan(desc, call, k) == plan
    cols = np.arange(d) if d <= 512 else edge_columns(d, n_random=48, seed=index)
    ci = torch.as_tensor(cols, device=DEV)
    xs, Ws, Ms = to_np64(x), to_np64(W[:, ci]), masks[:, :, ci].cpu().numpy()
    Wp = api.mglu_pack_weights(desc, W)
    tol = TOL[x.dtype]
    if call == "linear":
        out = api.mglu_linear_forward(desc, x, Wp)
        assert rel_err(to_np64(out[:, ci]), oracle.linear_forward(xs, Ws)) <= tol
        return
    if call == "swiglu":
        _, Wv, _ = synth.make_inputs(h, d, 1, 1, dtype=dname, seed=index + 1000, device=DEV)
        out = api.swiglu_forward(desc, x, Wp, api.mglu_pack_weights(desc, Wv))
        assert rel_err(to_np64(out[:, ci]), oracle.swiglu_forward(xs, Ws, to_np64(Wv[:, ci]))) <= tol
        return
    if call == "forward_routed":
        route = _route_weights(T, n_m, index, k)
        out = api.mglu_forward_routed(desc, x, Wp, api.mglu_pack_masks_planar(desc, masks),
                                      torch.as_tensor(route, device=DEV), k)
        assert rel_err(to_np64(out[:, ci]), oracle.mglu_forward_variant(xs, Ws, Ms, route=route)) <= tol
        return
    Mp = api.mglu_pack_masks(desc, masks)
    if call == "forward":
        out = api.mglu_forward(desc, x, Wp, Mp)
        assert rel_err(to_np64(out[:, ci]), oracle.mglu_forward(xs, Ws, Ms)) <= tol
    elif call == "forward_variant":
        var = dict(VARIATIONS[index % len(VARIATIONS)])
        route = _route_weights(T, n_m, index) if var.pop("route", False) else None
        out = api.mglu_forward_variant(desc, x, Wp, Mp, route_weights=None if route is None else
                                       torch.as_tensor(route, device=DEV), **var)
        ref = oracle.mglu_forward_variant(xs, Ws, Ms, route=route, **var)
        assert rel_err(to_np64(out[:, ci]), ref) <= tol
    else:
        t, gate, value = api.mglu_projections(desc, x, Wp, Mp)
        _, og, ov = oracle.mglu_forward(xs, Ws, Ms, return_projections=True)
        dense = xs @ Ws
        # fp32 sums of h products: accumulation error ~ sqrt(h) 2^-24 relative to the largest sum
        bound = 1e-5 * np.abs(dense).max()
        assert np.abs(to_np64(t[:, ci]) - dense).max() <= bound
        for i in range(n_m):
            assert np.abs(to_np64(gate[i][:, ci]) - og[i]).max() <= bound
            assert np.abs(to_np64(value[i][:, ci]) - ov[i]).max() <= bound
