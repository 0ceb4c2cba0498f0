"""Are the oracle's pins sharp?  A battery of the same kinds of checks as tests/test_oracle_pins.py
(closed forms, invariants, library special case, exact-rational brute force) is run against the
oracle -- it must pass -- and against deliberately wrong variants of Eq. 3 written here in numpy --
each must fail at least one check.  The mistakes are planted in these CPU variants only.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import mglu_oracle as oracle


def _swish(z, beta=1.0):
    return z / (1.0 + np.exp(-beta * z))


def make_variant(kind):
    """Eq. 3 in numpy with one planted mistake (kind=None: none)."""
    def f(x, W, M):
        x, W = np.asarray(x, np.float64), np.asarray(W, np.float64)
        M = np.asarray(M).astype(np.float64)
        n_m = M.shape[0]
        out = np.zeros((x.shape[0], W.shape[1]))
        for i in range(n_m):
            Mi = M[i]
            if kind == "first_mask_for_all":
                Mi = M[0]
            if kind == "mask_shifted_one_row":
                Mi = np.roll(Mi, 1, axis=0)
            if kind == "mask_transposed" and Mi.shape[0] == Mi.shape[1]:
                Mi = Mi.T
            gate_w, value_w = W * Mi, W * (1.0 - Mi)
            if kind == "value_not_complemented":
                value_w = W * Mi
            if kind == "value_is_dense":
                value_w = W
            xs = x[:, :-1] if kind == "drops_last_k" and x.shape[1] > 1 else x
            gw = gate_w[:-1] if kind == "drops_last_k" and x.shape[1] > 1 else gate_w
            vw = value_w[:-1] if kind == "drops_last_k" and x.shape[1] > 1 else value_w
            gate, value = xs @ gw, xs @ vw
            if kind == "gate_value_swapped":
                gate, value = value, gate
            if kind == "sigmoid_gate":
                g = 1.0 / (1.0 + np.exp(-gate))
            elif kind == "swish_beta":
                g = _swish(gate, 1.702)
            elif kind == "relu_gate":
                g = np.maximum(gate, 0.0)
            else:
                g = _swish(gate)
            term = g * value
            if kind == "value_sign":
                term = -term
            out += term
        if kind == "mean_over_masks":
            out /= n_m
        return out
    return f


MUTANTS = ["gate_value_swapped", "mean_over_masks", "swish_beta", "sigmoid_gate", "relu_gate",
           "first_mask_for_all", "mask_shifted_one_row", "mask_transposed", "value_not_complemented",
           "value_is_dense", "drops_last_k", "value_sign"]


def battery(f):
    """Names of the checks `f` fails (empty list = all pass)."""
    failed = []

    def check(name, ok):
        if not ok:
            failed.append(name)

    def close(a, b, rtol=1e-10):
        return np.max(np.abs(np.asarray(a) - np.asarray(b))) <= rtol * max(np.max(np.abs(b)), 1e-300)

    rng = np.random.default_rng(7)
    # hand-worked 2x2 (tests/golden/mglu_2x2_closed_form.txt)
    x = np.array([[1.0, 2.0]]); W = np.array([[1.0, -1.0], [0.5, 2.0]]); M = np.array([[[1, 0], [0, 1]]], np.uint8)
    check("closed_form_2x2", close(f(x, W, M)[0], [1 / (1 + math.exp(-1)), -4 / (1 + math.exp(-4))]))
    check("closed_form_2x2_complement", close(f(x, W, 1 - M)[0], [1 / (1 + math.exp(-1)), -4 / (1 + math.e)]))
    # single mask = SwiGLU through torch
    x = rng.standard_normal((3, 24)); W = rng.standard_normal((24, 24)) * 0.3
    M = (rng.random((1, 24, 24)) < 0.5).astype(np.uint8)
    xt, Wt, Mt = torch.from_numpy(x), torch.from_numpy(W), torch.from_numpy(M[0]).double()
    ref = (torch.nn.functional.silu(xt @ (Wt * Mt)) * (xt @ (Wt * (1 - Mt)))).numpy()
    check("single_mask_is_swiglu", close(f(x, W, M), ref))
    # additivity over masks, duplicates
    M3 = (rng.random((3, 24, 24)) < 0.5).astype(np.uint8)
    parts = sum(make_variant(None)(x, W, M3[i:i + 1]) for i in range(3))
    check("sum_over_masks", close(f(x, W, M3), parts))
    # degenerate masks and inputs
    ones = np.ones((1, 24, 24), np.uint8)
    check("all_gate_zero", np.all(f(x, W, ones) == 0.0))
    check("all_value_zero", np.all(f(x, W, 1 - ones) == 0.0))
    xh = np.zeros((1, 24)); xh[0, 23] = 2.5
    check("one_hot_zero", np.all(f(xh, W, M3) == 0.0))
    # two-hot closed form (rows 0 and 23: exercises the first and the last k)
    x2 = np.zeros((1, 24)); x2[0, 0] = x2[0, 23] = 1.0
    exp2 = np.zeros(24)
    for j in range(24):
        for i in range(3):
            g = W[0, j] * M3[i, 0, j] + W[23, j] * M3[i, 23, j]
            v = W[0, j] * (1 - M3[i, 0, j]) + W[23, j] * (1 - M3[i, 23, j])
            exp2[j] += g / (1 + math.exp(-g)) * v
    check("two_hot_closed_form", close(f(x2, W, M3)[0], exp2))
    # exact-rational brute force on a tiny shape
    xi = rng.integers(-6, 7, size=(2, 4)); Wi = rng.integers(-6, 7, size=(4, 3))
    Mb = rng.integers(0, 2, size=(2, 4, 3)).astype(np.uint8)
    expect = np.zeros((2, 3))
    for tau in range(2):
        for j in range(3):
            for i in range(2):
                gate = sum(Fraction(int(xi[tau, k]), 4) * Fraction(int(Wi[k, j]), 8) for k in range(4) if Mb[i, k, j])
                value = sum(Fraction(int(xi[tau, k]), 4) * Fraction(int(Wi[k, j]), 8) for k in range(4) if not Mb[i, k, j])
                expect[tau, j] += float(gate) / (1 + math.exp(-float(gate))) * float(value)
    check("brute_force", close(f(xi / 4.0, Wi / 8.0, Mb), expect, rtol=1e-12))
    return failed


def test_oracle_passes_the_battery():
    assert battery(oracle.mglu_forward) == []


def test_unmutated_variant_passes_the_battery():
    assert battery(make_variant(None)) == []


@pytest.mark.parametrize("kind", MUTANTS)
def test_every_planted_mistake_is_caught(kind):
    failed = battery(make_variant(kind))
    assert failed, "no check notices the mistake '%s'" % kind
