"""The C-ABI library loads, exports every symbol the header declares, and rejects bad
arguments with error codes before touching the GPU (no compute calls here)."""
import ctypes
import os
import re

import pytest

from paper_2506_23225_amd import _lib, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    build.build(force=False)
    return _lib.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "mglu.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b((?:mglu|swiglu)_[a-z_0-9]+)\s*\(", header))
    assert declared == set(_lib.SIGNATURES), declared ^ set(_lib.SIGNATURES)
    for name in declared:
        assert hasattr(lib, name), name


def test_sizes_follow_the_memory_model(lib):
    d = _lib.MgluDesc(1, 2048, 8192, 1, _lib.MGLU_BF16, _lib.MGLU_W_KN)
    assert lib.mglu_packed_weight_bytes(d) == 32 * 2 ** 20     # one 16-bit matrix of the paper's Llama-1B example
    assert lib.mglu_packed_mask_bytes(d) == 2 * 2 ** 20        # one mask plane: 2 MiB
    for n_m, planes in ((2, 2), (3, 4), (4, 4), (5, 8), (8, 8)):
        d.n_masks = n_m
        assert lib.mglu_packed_mask_bytes(d) == planes * 2 * 2 ** 20
    # padding to 16 columns x 128 rows
    d = _lib.MgluDesc(1, 200, 50, 1, _lib.MGLU_F32, _lib.MGLU_W_KN)
    assert lib.mglu_packed_weight_bytes(d) == 256 * 64 * 4
    assert lib.mglu_packed_mask_bytes(d) == 256 * 64 // 8
    # scratch: only where the MFMA-tiled kernel runs a layer of more than 8 masks in two launches (more than 32 tokens)
    for dtype, n_m, T, want in ((_lib.MGLU_BF16, 16, 4096, 4096 * 14336 * 4), (_lib.MGLU_F16, 9, 33, 33 * 14336 * 4),
                                (_lib.MGLU_BF16, 8, 4096, 0), (_lib.MGLU_BF16, 16, 16, 0), (_lib.MGLU_BF16, 16, 32, 0),
                                (_lib.MGLU_F32, 16, 4096, 0)):
        assert lib.mglu_workspace_bytes(_lib.MgluDesc(T, 4096, 14336, n_m, dtype, _lib.MGLU_W_KN)) == want


def test_bad_arguments_are_reported_not_launched(lib):
    ok = _lib.MgluDesc(1, 256, 64, 2, _lib.MGLU_BF16, _lib.MGLU_W_KN)
    fake = ctypes.c_void_p(0x1000)
    INVALID, UNSUPPORTED, WORKSPACE = 1, 2, 3

    def fwd(desc, x=fake, w=fake, m=fake, out=fake):
        return lib.mglu_forward(desc, x, w, m, out, None, 0, None)

    assert fwd(None) == INVALID
    assert fwd(ok, x=None) == INVALID and b"x_dev" in lib.mglu_last_error()
    assert fwd(ok, out=ctypes.c_void_p(0x1004)) == INVALID and b"aligned" in lib.mglu_last_error()
    for field, value, code in (("tokens", 0, INVALID), ("d_model", 0, INVALID), ("d_ff", -1, INVALID),
                               ("n_masks", 0, INVALID), ("n_masks", 17, UNSUPPORTED),
                               ("dtype", 7, INVALID), ("w_layout", 2, INVALID), ("d_model", 100, UNSUPPORTED)):
        bad = _lib.MgluDesc(1, 256, 64, 2, _lib.MGLU_BF16, _lib.MGLU_W_KN)
        setattr(bad, field, value)
        assert fwd(bad) == code, (field, value, lib.mglu_last_error())
    assert lib.mglu_forward_bool(ok, fake, fake, fake, fake, fake, 16, None) == WORKSPACE
    two_launches = _lib.MgluDesc(64, 256, 64, 16, _lib.MGLU_BF16, _lib.MGLU_W_KN)
    assert fwd(two_launches) == WORKSPACE and b"mglu_workspace_bytes" in lib.mglu_last_error()
    assert lib.mglu_forward(two_launches, fake, fake, fake, fake, fake, 64 * 64 * 4 - 1, None) == WORKSPACE
    # the allocation-free variant refuses layers beyond its static staging array, and bad pointers, before any GPU call
    big = _lib.MgluDesc(1, 4096, 14336, 8, _lib.MGLU_BF16, _lib.MGLU_W_KN)
    assert lib.mglu_forward_bool_static(big, fake, fake, fake, fake, None) == WORKSPACE
    assert b"static scratch" in lib.mglu_last_error()
    assert lib.mglu_forward_bool_static(ok, fake, None, fake, fake, None) == INVALID
    assert lib.mglu_forward_bool(ok, fake, fake, fake, None, fake, 1 << 30, None) == INVALID   # out checked before any launch
    assert lib.mglu_pack_masks(ok, None, fake, None) == INVALID
    assert lib.mglu_pack_weights(ok, fake, None, None) == INVALID
    assert lib.mglu_stream_read(fake, 24, fake, None) == INVALID
    assert lib.mglu_packed_mask_bytes(None) == 0
    assert lib.mglu_status_string(2) == b"unsupported"
