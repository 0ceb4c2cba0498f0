"""Loads ``libmglu.so`` (the C ABI of include/mglu.h) through ctypes.

There is no fallback: if the library has not been built, loading raises.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmglu.so")

MGLU_OK = 0
MGLU_F32, MGLU_BF16, MGLU_F16 = 0, 1, 2
MGLU_W_KN, MGLU_W_NK = 0, 1


class MgluDesc(ctypes.Structure):
    _fields_ = [("tokens", ctypes.c_int32), ("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32),
                ("n_masks", ctypes.c_int32), ("dtype", ctypes.c_int), ("w_layout", ctypes.c_int)]


class MgluVariant(ctypes.Structure):
    _fields_ = [("gate", ctypes.c_int), ("mask_use", ctypes.c_int), ("route_weights_dev", ctypes.c_void_p)]


MGLU_CALL = {"forward": 0, "forward_variant": 1, "projections": 2, "linear": 3, "swiglu": 4, "forward_routed": 5}
MGLU_GATE = {"swish": 0, "gelu": 1, "relu": 2}
MGLU_MASK_USE = {"both": 0, "dense_gate": 1, "dense_value": 2, "none": 3}

# every symbol include/mglu.h declares: name -> (restype, argtypes)
_P = ctypes.c_void_p
_D = ctypes.POINTER(MgluDesc)
_SZ = ctypes.c_size_t
SIGNATURES = {
    "mglu_format_version": (ctypes.c_int, []),
    "mglu_packed_weight_bytes": (_SZ, [_D]),
    "mglu_pack_weights": (ctypes.c_int, [_D, _P, _P, _P]),
    "mglu_packed_mask_bytes": (_SZ, [_D]),
    "mglu_pack_masks": (ctypes.c_int, [_D, _P, _P, _P]),
    "mglu_workspace_bytes": (_SZ, [_D]),
    "mglu_forward": (ctypes.c_int, [_D, _P, _P, _P, _P, _P, _SZ, _P]),
    "mglu_forward_bool_workspace_bytes": (_SZ, [_D]),
    "mglu_forward_bool": (ctypes.c_int, [_D, _P, _P, _P, _P, _P, _SZ, _P]),
    "mglu_forward_bool_static": (ctypes.c_int, [_D, _P, _P, _P, _P, _P]),
    "mglu_projections": (ctypes.c_int, [_D, _P, _P, _P, _P, _P, _P, _P, _SZ, _P]),
    "mglu_forward_variant": (ctypes.c_int, [_D, ctypes.POINTER(MgluVariant), _P, _P, _P, _P, _P, _SZ, _P]),
    "mglu_route_topk": (ctypes.c_int, [_D, _P, _P, ctypes.c_int, _P, _P]),
    "mglu_linear_forward": (ctypes.c_int, [_D, _P, _P, _P, _P, _SZ, _P]),
    "mglu_ffn_forward": (ctypes.c_int, [_D, ctypes.POINTER(MgluVariant), _P, _P, _P, _P, _P, _P, _P, _SZ, _P]),
    "swiglu_forward": (ctypes.c_int, [_D, _P, _P, _P, _P, _P, _SZ, _P]),
    "mglu_stream_read": (ctypes.c_int, [_P, _SZ, _P, _P]),
    "mglu_describe_plan": (ctypes.c_int, [_D, ctypes.c_int, ctypes.c_int, ctypes.c_char_p, _SZ]),
    "mglu_packed_mask_bytes_planar": (_SZ, [_D]),
    "mglu_pack_masks_planar": (ctypes.c_int, [_D, _P, _P, _P]),
    "mglu_forward_routed": (ctypes.c_int, [_D, _P, _P, _P, _P, ctypes.c_int, ctypes.c_int, _P, _P]),
    "mglu_last_error": (ctypes.c_char_p, []),
    "mglu_status_string": (ctypes.c_char_p, [ctypes.c_int]),
}

_lib = None


def load(path=None):
    """The loaded library, with argument types set.  Raises if libmglu.so is missing.

    `path` (first call only) loads another build of the same ABI instead, e.g. one compiled with
    other tuning macros for an experiment; the product never passes it."""
    global _lib
    if _lib is None:
        path = path or LIB_PATH
        if not os.path.exists(path):
            raise RuntimeError(
                "%s is missing: build it with `python -m paper_2506_23225_amd.build` "
                "(there is no fallback path)" % path)
        lib = ctypes.CDLL(path)
        for name, (restype, argtypes) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = restype
            fn.argtypes = argtypes
        _lib = lib
    return _lib
