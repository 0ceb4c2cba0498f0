"""Host-only checks of the plan query: the descriptor grid of tests/plans.py reaches every kernel
instantiation compiled into libmglu.so (so the GPU suite's one-parity-case-per-plan covers every code path
the launchers can select), and the benchmark configurations run the kernels the reports name."""
import re
import shutil
import subprocess

import pytest
import torch

from paper_2506_23225_amd import _lib, api, build
from tests import plans


@pytest.fixture(scope="module")
def lib():
    build.build(force=False)
    return _lib.load()


def _compiled_kernels():
    """MGLU kernel instantiations in the library's own symbol table (the host-side launch stubs)."""
    nm = shutil.which("nm") or shutil.which("llvm-nm", path="/opt/rocm/llvm/bin")
    if not nm:
        pytest.skip("no nm to list the library's symbols with")
    out = subprocess.run([nm, "-C", _lib.LIB_PATH], capture_output=True, text=True, check=True).stdout
    names = set()
    for line in out.splitlines():
        m = re.search(r"__device_stub__((?:stream_resident|stream_panel|stream_routed|prefill)_kernel<.*>)\(", line)
        if m:
            names.add(m.group(1).replace("mglu::", ""))
    return names


def test_grid_reaches_every_compiled_instantiation(lib):
    compiled = _compiled_kernels()
    # a plan is a kernel instantiation, plus " twice" where a layer of more than 8 masks runs it once per half
    reached = {name.removesuffix(" twice") for name in plans.enumerate_plans()}
    assert any(name.endswith(" twice") for name in plans.enumerate_plans())
    assert len(compiled) > 100
    assert reached - compiled == set(), "the plan query names kernels that are not in the library"
    assert compiled - reached == set(), "compiled but selected by no descriptor of the grid: dead, or extend the grid"


@pytest.mark.parametrize("T,h,d,n_m,expect", [
    (1, 2048, 5632, 4, "stream_resident_kernel<Bf16Traits, 4, 0, 2, true>"),
    (1, 4096, 14336, 8, "stream_resident_kernel<Bf16Traits, 8, 0, 2, false>"),
    (1, 4096, 14336, 16, "stream_resident_kernel<Bf16Traits, 16, 0, 2, false>"),
    (1, 8192, 28672, 2, "stream_resident_kernel<Bf16Traits, 2, 0, 2, false>"),
    (32, 8192, 28672, 1, "stream_panel_kernel<Bf16Traits, 1, 2, 0, 8, 1, 2>"),
    (32, 8192, 28672, 4, "stream_panel_kernel<Bf16Traits, 4, 2, 0, 8, 1, 2>"),
    (4096, 4096, 14336, 4, "prefill_kernel<Bf16Traits, 4, 1, 8, 0, 2, 8>"),
    (4096, 4096, 14336, 16, "prefill_kernel<Bf16Traits, 8, 1, 4, 0, 2, 8> twice"),
    (2048, 8192, 28672, 2, "prefill_kernel<Bf16Traits, 2, 1, 8, 0, 2, 8>"),
    (80, 136, 28672, 4, "prefill_kernel<Bf16Traits, 4, 1, 6, 0, 2, 8>"),
    (390, 136, 28672, 4, "prefill_kernel<Bf16Traits, 4, 1, 8, 0, 3, 4>"),
])
def test_benchmark_shapes_run_the_named_kernels(lib, T, h, d, n_m, expect):
    assert api.mglu_describe_plan(api.make_desc(T, h, d, n_m, torch.bfloat16)) == expect


def test_describe_plan_rejects_bad_arguments(lib):
    import ctypes
    ok = _lib.MgluDesc(1, 256, 64, 2, _lib.MGLU_BF16, _lib.MGLU_W_KN)
    buf = ctypes.create_string_buffer(8)
    assert lib.mglu_describe_plan(ok, 0, 0, buf, 8) == 0 and buf.value == b"stream_"   # truncated, NUL-terminated
    assert lib.mglu_describe_plan(ok, 9, 0, buf, 8) == 1
    assert lib.mglu_describe_plan(ok, 0, 0, None, 8) == 1
    assert lib.mglu_describe_plan(None, 0, 0, buf, 8) == 1
    bad = _lib.MgluDesc(1, 100, 64, 2, _lib.MGLU_BF16, _lib.MGLU_W_KN)
    assert lib.mglu_describe_plan(bad, 0, 0, buf, 8) == 2
    assert lib.mglu_describe_plan(ok, 5, 3, buf, 8) == 1          # routed: k beyond n_masks
    many = _lib.MgluDesc(17, 256, 64, 2, _lib.MGLU_BF16, _lib.MGLU_W_KN)
    assert lib.mglu_describe_plan(many, 5, 1, buf, 8) == 2        # routed: more than 16 tokens
