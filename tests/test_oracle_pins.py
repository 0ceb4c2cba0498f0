"""Pins for the fp64 CPU oracle (no GPU needed).

Each test checks the oracle against something other than itself: a closed
form, an invariant of Eq. 2 / Eq. 3, a special case that reduces to a library
routine, or brute force in exact rational arithmetic on a tiny shape.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import mglu_oracle as oracle

RTOL = 1e-12


def _rand(T, h, d, n_m, seed=0, p=0.5, w_std=0.02):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, h))
    W = rng.standard_normal((h, d)) * w_std
    M = (rng.random((n_m, h, d)) < p).astype(np.uint8)
    return x, W, M


def _close(a, b, rtol=RTOL):
    scale = max(np.max(np.abs(b)), 1e-300)
    assert np.max(np.abs(a - b)) <= rtol * scale, np.max(np.abs(a - b)) / scale


def _read_golden(path):
    vals = {}
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *rest = line.split()
            vals[key] = [float(v) for v in rest]
    return vals


def test_hand_worked_2x2(golden_dir):
    """Closed form worked by hand from Eq. 2 (tests/golden/mglu_2x2_closed_form.txt)."""
    g = _read_golden(os.path.join(golden_dir, "mglu_2x2_closed_form.txt"))
    x = np.array([[1.0, 2.0]])
    W = np.array([[1.0, -1.0], [0.5, 2.0]])
    M = np.array([[[1, 0], [0, 1]]], dtype=np.uint8)
    np.testing.assert_allclose(oracle.mglu_forward(x, W, M)[0], g["out"], rtol=1e-15)
    np.testing.assert_allclose(oracle.mglu_forward(x, W, 1 - M)[0], g["out_complemented_mask"], rtol=1e-15)


def test_partition_sums_to_dense_projection():
    """gate_i + value_i = xW for every mask, since M + Mbar = 1 (Eq. 2)."""
    x, W, M = _rand(3, 67, 45, 4, seed=1)
    out, gate, value = oracle.mglu_forward(x, W, M, return_projections=True)
    dense = x @ W  # numpy fp64 matmul, independent of the oracle's loops
    for i in range(M.shape[0]):
        _close(gate[i] + value[i], dense)
    # the output is the swish-gated sum of those projections (Eq. 3)
    ref = sum((gate[i] / (1 + np.exp(-gate[i]))) * value[i] for i in range(M.shape[0]))
    _close(out, ref)


def test_projections_match_library_matmul():
    """Each branch equals a library fp64 matmul on the materialised masked matrix."""
    x, W, M = _rand(2, 40, 33, 3, seed=2)
    _, gate, value = oracle.mglu_forward(x, W, M, return_projections=True)
    for i in range(3):
        _close(gate[i], x @ (W * M[i]))
        _close(value[i], x @ (W * (1 - M[i])))


def test_single_mask_is_swiglu_via_torch():
    """n_m = 1 is Eq. 1 with W_g = W*M, W_v = W*(1-M): checked with torch CPU fp64 matmul + silu."""
    x, W, M = _rand(5, 96, 80, 1, seed=3)
    xt, Wt, Mt = torch.from_numpy(x), torch.from_numpy(W), torch.from_numpy(M[0]).double()
    ref = torch.nn.functional.silu(xt @ (Wt * Mt)) * (xt @ (Wt * (1 - Mt)))
    _close(oracle.mglu_forward(x, W, M), ref.numpy())
    # and the oracle's own two-matrix GLU entry agrees with the same library routine
    _close(oracle.swiglu_forward(x, W * M[0], W * (1 - M[0])), ref.numpy())


def test_swiglu_entry_against_torch():
    rng = np.random.default_rng(4)
    x, Wg, Wv = rng.standard_normal((3, 50)), rng.standard_normal((50, 21)), rng.standard_normal((50, 21))
    ref = torch.nn.functional.silu(torch.from_numpy(x @ Wg)) * torch.from_numpy(x @ Wv)
    _close(oracle.swiglu_forward(x, Wg, Wv), ref.numpy())


def test_all_gate_and_all_value_masks_give_exact_zero():
    """M = 1: value branch is empty; M = 0: gate is 0 and swish(0) = 0.  Exact."""
    x, W, _ = _rand(2, 31, 17, 1, seed=5)
    ones = np.ones((1, 31, 17), dtype=np.uint8)
    assert np.all(oracle.mglu_forward(x, W, ones) == 0.0)
    assert np.all(oracle.mglu_forward(x, W, 1 - ones) == 0.0)
    # as extra routes they add nothing
    _, _, M = _rand(2, 31, 17, 2, seed=6)
    base = oracle.mglu_forward(x, W, M)
    both = oracle.mglu_forward(x, W, np.concatenate([M, ones, 1 - ones]))
    assert np.array_equal(base, both)


def test_one_hot_input_gives_exact_zero():
    """x = c e_k: each weight element feeds only one branch, so one factor of every product is 0."""
    _, W, M = _rand(1, 23, 19, 4, seed=7)
    for k in (0, 11, 22):
        x = np.zeros((1, 23))
        x[0, k] = -3.25
        assert np.all(oracle.mglu_forward(x, W, M) == 0.0)


def test_two_hot_input_closed_form():
    """x = e_a + e_b: out[j] = sum_i swish(W_aj m_a + W_bj m_b) * (W_aj (1-m_a) + W_bj (1-m_b))."""
    _, W, M = _rand(1, 16, 29, 3, seed=8)
    a, b = 2, 9
    x = np.zeros((1, 16))
    x[0, a] = x[0, b] = 1.0
    expect = np.zeros(29)
    for j in range(29):
        for i in range(3):
            g = W[a, j] * M[i, a, j] + W[b, j] * M[i, b, j]
            v = W[a, j] * (1 - M[i, a, j]) + W[b, j] * (1 - M[i, b, j])
            expect[j] += g / (1 + math.exp(-g)) * v
    _close(oracle.mglu_forward(x, W, M)[0], expect)
    # nonzero exactly where some mask separates the two elements
    differs = (M[:, a, :] != M[:, b, :]).any(axis=0)
    assert np.array_equal(oracle.mglu_forward(x, W, M)[0] != 0.0, differs)


def test_additivity_duplicates_and_permutation():
    """Eq. 3 is a plain sum over routes."""
    x, W, M = _rand(3, 48, 37, 4, seed=9)
    full = oracle.mglu_forward(x, W, M)
    parts = sum(oracle.mglu_forward(x, W, M[i:i + 1]) for i in range(4))
    _close(full, parts)
    _close(oracle.mglu_forward(x, W, M[[2, 0, 3, 1]]), full)
    one = oracle.mglu_forward(x, W, M[:1])
    _close(oracle.mglu_forward(x, W, np.concatenate([M[:1], M[:1]])), 2 * one)


def test_rows_are_independent():
    x, W, M = _rand(4, 33, 21, 2, seed=10)
    full = oracle.mglu_forward(x, W, M)
    for tau in range(4):
        assert np.array_equal(oracle.mglu_forward(x[tau:tau + 1], W, M)[0], full[tau])


@pytest.mark.parametrize("T,h,d,n_m", [(1, 1, 1, 1), (2, 3, 2, 2), (2, 4, 3, 2), (1, 5, 3, 3)])
def test_brute_force_exact_rationals(T, h, d, n_m):
    """Triple loop in exact rational arithmetic; only exp() is floating point."""
    rng = np.random.default_rng(100 + h * d + n_m)
    xi = rng.integers(-8, 9, size=(T, h))
    Wi = rng.integers(-8, 9, size=(h, d))
    M = rng.integers(0, 2, size=(n_m, h, d)).astype(np.uint8)
    x, W = xi / 4.0, Wi / 16.0  # exactly representable
    expect = np.zeros((T, d))
    for tau in range(T):
        for j in range(d):
            acc = 0.0
            for i in range(n_m):
                gate = sum(Fraction(int(xi[tau, k]), 4) * Fraction(int(Wi[k, j]), 16)
                           for k in range(h) if M[i, k, j] == 1)
                value = sum(Fraction(int(xi[tau, k]), 4) * Fraction(int(Wi[k, j]), 16)
                            for k in range(h) if M[i, k, j] == 0)
                g = float(gate)
                acc += g / (1.0 + math.exp(-g)) * float(value)
            expect[tau, j] = acc
    got = oracle.mglu_forward(x, W, M)
    assert np.max(np.abs(got - expect)) <= 1e-14 * max(1.0, np.max(np.abs(expect)))


def test_complementing_the_mask_changes_the_result():
    """Gate and value are not interchangeable: swapping M and 1-M gives sum swish(value)*gate."""
    x, W, M = _rand(2, 40, 30, 2, seed=11)
    _, gate, value = oracle.mglu_forward(x, W, M, return_projections=True)
    swapped = oracle.mglu_forward(x, W, 1 - M)
    ref = sum(value[i] / (1 + np.exp(-value[i])) * gate[i] for i in range(2))
    _close(swapped, ref)
    assert np.max(np.abs(swapped - oracle.mglu_forward(x, W, M))) > 1e-3 * np.max(np.abs(ref))


def test_small_input_regime_is_quadratic():
    """swish(z) ~ z/2 near 0, so out(alpha x)/alpha^2 -> (1/2) sum_i gate_i value_i."""
    x, W, M = _rand(2, 64, 25, 3, seed=12)
    _, gate, value = oracle.mglu_forward(x, W, M, return_projections=True)
    limit = 0.5 * sum(gate[i] * value[i] for i in range(3))
    alpha = 1e-6
    _close(oracle.mglu_forward(alpha * x, W, M) / alpha ** 2, limit, rtol=1e-5)


def test_swish_values():
    """g(z) = z sigmoid(z) with beta = 1, read through a 1x1 layer: gate = z, value = 1."""
    for z in (-20.0, -1.0, 0.0, 0.5, 3.0, 30.0):
        x = np.array([[z, 1.0]])
        W = np.array([[1.0], [1.0]])
        M = np.array([[[1], [0]]], dtype=np.uint8)
        expect = z / (1.0 + math.exp(-z))
        assert abs(oracle.mglu_forward(x, W, M)[0, 0] - expect) <= 1e-15 * max(1.0, abs(expect))


def test_empty_shapes():
    assert oracle.mglu_forward(np.zeros((0, 4)), np.zeros((4, 3)), np.zeros((1, 4, 3), np.uint8)).shape == (0, 3)
    out = oracle.mglu_forward(np.ones((2, 4)), np.ones((4, 3)), np.zeros((0, 4, 3), np.uint8))
    assert out.shape == (2, 3) and np.all(out == 0.0)


def test_bf16_inputs_are_widened_exactly():
    """bf16-rounded inputs reach the oracle unchanged."""
    xt = torch.randn(2, 32, generator=torch.Generator().manual_seed(0)).to(torch.bfloat16)
    Wt = (torch.randn(32, 16, generator=torch.Generator().manual_seed(1)) * 0.02).to(torch.bfloat16)
    M = np.ones((1, 32, 16), np.uint8)
    M[0, ::2] = 0
    a = oracle.mglu_forward(xt.double().numpy(), Wt.double().numpy(), M)
    b = oracle.mglu_forward(xt.float().numpy(), Wt.float().numpy(), M)
    assert np.array_equal(a, b)
