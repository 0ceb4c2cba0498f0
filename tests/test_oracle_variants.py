"""Pins for the oracle's variant entry points (appendix: other gate functions, partial-mask
ablations, Top-K routing) and for the output projection.  No GPU needed."""
import math

import numpy as np
import pytest
import torch

from oracle import mglu_oracle as oracle


def _rand(T, h, d, n_m, seed=0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((T, h)), rng.standard_normal((h, d)) * 0.3,
            (rng.random((n_m, h, d)) < 0.5).astype(np.uint8))


def _close(a, b, rtol=1e-12):
    assert np.max(np.abs(a - b)) <= rtol * max(np.max(np.abs(b)), 1e-300)


def test_default_variant_is_eq3():
    x, W, M = _rand(3, 20, 14, 3, seed=1)
    assert np.array_equal(oracle.mglu_forward_variant(x, W, M), oracle.mglu_forward(x, W, M))
    ones = np.ones((3, 3))
    assert np.array_equal(oracle.mglu_forward_variant(x, W, M, route=ones), oracle.mglu_forward(x, W, M))


@pytest.mark.parametrize("gate,fn", [
    ("gelu", lambda z: torch.nn.functional.gelu(z)),          # exact (erf) GELU, library routine
    ("relu", lambda z: torch.relu(z)),
    ("swish", lambda z: torch.nn.functional.silu(z)),
])
def test_gate_functions_against_torch(gate, fn):
    x, W, M = _rand(4, 32, 18, 2, seed=2)
    xt, Wt = torch.from_numpy(x), torch.from_numpy(W)
    ref = sum(fn(xt @ (Wt * torch.from_numpy(M[i]).double())) * (xt @ (Wt * (1 - torch.from_numpy(M[i]).double())))
              for i in range(2)).numpy()
    _close(oracle.mglu_forward_variant(x, W, M, gate=gate), ref)


def test_gate_function_values():
    """g read through a 1x1 layer: gate = z, value = 1."""
    for z in (-3.0, -0.5, 0.0, 0.7, 2.5):
        x = np.array([[z, 1.0]]); W = np.array([[1.0], [1.0]]); M = np.array([[[1], [0]]], np.uint8)
        assert abs(oracle.mglu_forward_variant(x, W, M, gate="relu")[0, 0] - max(z, 0.0)) < 1e-15
        gelu = 0.5 * z * (1.0 + math.erf(z / math.sqrt(2.0)))
        assert abs(oracle.mglu_forward_variant(x, W, M, gate="gelu")[0, 0] - gelu) < 1e-15


def test_partial_mask_ablations():
    x, W, M = _rand(3, 28, 16, 2, seed=3)
    dense = x @ W
    sw = lambda z: z / (1 + np.exp(-z))
    gates = [x @ (W * M[i]) for i in range(2)]
    values = [x @ (W * (1 - M[i])) for i in range(2)]
    _close(oracle.mglu_forward_variant(x, W, M, mask_use="dense_gate"), sum(sw(dense) * v for v in values))
    _close(oracle.mglu_forward_variant(x, W, M, mask_use="dense_value"), sum(sw(g) * dense for g in gates))
    _close(oracle.mglu_forward_variant(x, W, M, mask_use="none"), 2 * sw(dense) * dense)
    # the ablations differ from the masked layer
    full = oracle.mglu_forward(x, W, M)
    for use in ("dense_gate", "dense_value", "none"):
        assert np.max(np.abs(oracle.mglu_forward_variant(x, W, M, mask_use=use) - full)) > 1e-3


def test_route_weights_scale_routes():
    x, W, M = _rand(2, 24, 12, 3, seed=4)
    route = np.array([[0.2, 0.0, 0.8], [0.0, 1.0, 0.0]])
    singles = [oracle.mglu_forward(x, W, M[i:i + 1]) for i in range(3)]
    ref = sum(route[:, i:i + 1] * singles[i] for i in range(3))
    _close(oracle.mglu_forward_variant(x, W, M, route=route), ref)


def test_router_topk_against_torch():
    rng = np.random.default_rng(5)
    x, Wr = rng.standard_normal((6, 40)), rng.standard_normal((40, 8))
    logits = torch.from_numpy(x @ Wr)
    # K = n_m: plain softmax (library routine)
    _close(oracle.route_topk(x, Wr, 8), torch.softmax(logits, dim=1).numpy())
    # K = 1: one-hot at the argmax
    w1 = oracle.route_topk(x, Wr, 1)
    assert np.array_equal(w1.argmax(axis=1), logits.argmax(dim=1).numpy()) and np.all(np.sort(w1, axis=1)[:, -1] == 1.0)
    # K = 3: torch.topk + softmax over the kept logits
    w3 = oracle.route_topk(x, Wr, 3)
    vals, idx = torch.topk(logits, 3, dim=1)
    ref = torch.zeros_like(logits).scatter(1, idx, torch.softmax(vals, dim=1)).numpy()
    _close(w3, ref)
    assert np.all((w3 > 0).sum(axis=1) == 3)
    np.testing.assert_allclose(w3.sum(axis=1), 1.0, rtol=1e-14)


def test_router_tie_goes_to_the_lower_index():
    x = np.ones((1, 2)); Wr = np.array([[1.0, 1.0, 0.5], [0.0, 0.0, 0.0]])
    assert np.array_equal(oracle.route_topk(x, Wr, 1), [[1.0, 0.0, 0.0]])


def test_linear_is_a_plain_matmul():
    rng = np.random.default_rng(6)
    a, W = rng.standard_normal((5, 37)), rng.standard_normal((37, 23))
    _close(oracle.linear_forward(a, W), a @ W)
    eye = np.eye(9)
    assert np.array_equal(oracle.linear_forward(a[:, :9], eye), a[:, :9])
