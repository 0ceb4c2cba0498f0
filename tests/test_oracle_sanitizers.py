"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only, no GPU).

tests/oracle_sanitize_driver.c is compiled together with oracle/mglu_oracle.c with
-fsanitize=address,undefined; it runs every oracle entry point on seeded inputs (ragged shapes, a
single token, 16 masks, an empty batch).  The sanitizers must stay silent and the results must equal
the regular oracle build's.
"""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import mglu_oracle as oracle

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    if not shutil.which("gcc"):
        pytest.skip("no gcc")
    exe = str(tmp_path_factory.mktemp("san") / "oracle_san")
    cmd = ["gcc", "-std=c99", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-Wall", "-Wextra", "-o", exe,
           os.path.join(HERE, "oracle_sanitize_driver.c"), "-lm"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0 and "sanitize" in res.stderr and "cannot find" in res.stderr:
        pytest.skip("sanitizer runtime not installed: " + res.stderr[-200:])
    assert res.returncode == 0, res.stderr
    return exe


@pytest.mark.parametrize("T,h,d,n_m,K,has_route", [
    (1, 8, 1, 1, 1, 0), (3, 200, 50, 3, 2, 1), (5, 264, 300, 16, 4, 1), (17, 136, 17, 5, 5, 0), (0, 16, 8, 2, 1, 0),
    (2, 1, 257, 8, 3, 1),
])
def test_oracle_is_clean_under_asan_ubsan(driver, tmp_path, T, h, d, n_m, K, has_route):
    rng = np.random.default_rng(T + h + d + n_m)
    x = rng.standard_normal((T, h))
    W = rng.standard_normal((h, d)) * 0.02
    W2 = rng.standard_normal((h, d)) * 0.02
    Wr = rng.standard_normal((h, n_m)) * 0.1
    route = rng.random((T, n_m))
    M = (rng.random((n_m, h, d)) < 0.5).astype(np.uint8)
    inp, outp = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(inp, "wb") as f:
        f.write(np.array([T, h, d, n_m, K, has_route], dtype=np.int64).tobytes())
        for a in (x, W, W2, Wr, route):
            f.write(np.ascontiguousarray(a, dtype=np.float64).tobytes())
        f.write(M.tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    env.pop("LD_PRELOAD", None)   # the sanitizer runtime has to come first in the program's own link order
    res = subprocess.run([driver, inp, outp], capture_output=True, text=True, env=env, timeout=120)
    assert res.returncode == 0, res.stderr[-2000:]
    assert "ERROR" not in res.stderr and "runtime error" not in res.stderr, res.stderr[-2000:]
    got = np.fromfile(outp, dtype=np.float64)
    Td = T * d
    parts = np.split(got, np.cumsum([Td, n_m * Td, n_m * Td, Td, Td, T * n_m]))
    if T == 0:
        assert got.size == 0
        return
    out, gate, value = oracle.mglu_forward(x, W, M, return_projections=True)
    want = [out, gate, value, oracle.swiglu_forward(x, W, W2),
            oracle.mglu_forward_variant(x, W, M, gate="gelu", mask_use="dense_value", route=route if has_route else None),
            oracle.route_topk(x, Wr, K), oracle.linear_forward(x, W)]
    for g, w in zip(parts, want):
        w = np.asarray(w).ravel()
        assert g.shape == w.shape
        assert np.max(np.abs(g - w)) <= 1e-13 * max(1.0, np.max(np.abs(w)))
