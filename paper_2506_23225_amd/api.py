"""Thin Python binding of libmglu: same names as the C ABI, argument marshalling only.

torch is used for device memory and the current HIP stream; every step of the
MGLU path runs in the library's kernels.  Tensors must live on the GPU and be
contiguous.
"""
import ctypes

import torch

from . import _lib
from ._lib import MgluDesc

_DTYPE = {torch.float32: _lib.MGLU_F32, torch.bfloat16: _lib.MGLU_BF16, torch.float16: _lib.MGLU_F16}
_LAYOUT = {"kn": _lib.MGLU_W_KN, "nk": _lib.MGLU_W_NK}


class MgluError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("libmglu status %d (%s): %s" % (
            status, _lib.load().mglu_status_string(status).decode(), message))
        self.status = status


def _check(status):
    if status != _lib.MGLU_OK:
        raise MgluError(status, _lib.load().mglu_last_error().decode())


def _stream(t):
    return torch.cuda.current_stream(t.device).cuda_stream


def _ptr(t, name):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must be a GPU tensor" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return t.data_ptr()


_TORCH_OF = {v: k for k, v in _DTYPE.items()}


def _expect(t, name, numel=None, dtype=None, min_bytes=None):
    """Cheap host-side checks of a tensor against the descriptor: the kernels trust the sizes they are given."""
    if t is None:
        return
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s has dtype %s, the descriptor says %s" % (name, t.dtype, dtype))
    if numel is not None and t.numel() != numel:
        raise ValueError("%s has %d elements, the descriptor says %d" % (name, t.numel(), numel))
    if min_bytes is not None and t.numel() * t.element_size() < min_bytes:
        raise ValueError("%s holds %d bytes, %d are needed" % (name, t.numel() * t.element_size(), min_bytes))


def _expect_layer(desc, x=None, out=None, W_packed=None, masks_packed=None, W=None, masks=None):
    dt = _TORCH_OF[desc.dtype]
    _expect(x, "x", desc.tokens * desc.d_model, dt)
    _expect(out, "out", desc.tokens * desc.d_ff, dt)
    _expect(W, "W", desc.d_model * desc.d_ff, dt)
    _expect(masks, "masks", desc.n_masks * desc.d_model * desc.d_ff, torch.uint8)
    if W_packed is not None:
        _expect(W_packed, "W_packed", min_bytes=mglu_packed_weight_bytes(desc))
    if masks_packed is not None:
        _expect(masks_packed, "masks_packed", min_bytes=mglu_packed_mask_bytes(desc))


def make_desc(tokens, d_model, d_ff, n_masks, dtype, w_layout="kn"):
    return MgluDesc(int(tokens), int(d_model), int(d_ff), int(n_masks), _DTYPE[dtype], _LAYOUT[w_layout])


def mglu_format_version():
    return _lib.load().mglu_format_version()


def mglu_packed_weight_bytes(desc):
    return _lib.load().mglu_packed_weight_bytes(desc)


def mglu_packed_mask_bytes(desc):
    return _lib.load().mglu_packed_mask_bytes(desc)


def mglu_workspace_bytes(desc):
    return _lib.load().mglu_workspace_bytes(desc)


def mglu_forward_bool_workspace_bytes(desc):
    return _lib.load().mglu_forward_bool_workspace_bytes(desc)


def mglu_pack_weights(desc, W, packed=None):
    """W [d_model,d_ff] ('kn') or [d_ff,d_model] ('nk') -> packed uint8 buffer."""
    _expect_layer(desc, W=W)
    if packed is None:
        packed = torch.empty(mglu_packed_weight_bytes(desc), dtype=torch.uint8, device=W.device)
    _expect(packed, "packed", min_bytes=mglu_packed_weight_bytes(desc))
    _check(_lib.load().mglu_pack_weights(desc, _ptr(W, "W"), _ptr(packed, "packed"), _stream(W)))
    return packed


def mglu_pack_masks(desc, masks, packed=None):
    """masks uint8/bool [n_masks,d_model,d_ff] ('kn') or [n_masks,d_ff,d_model] ('nk') -> packed buffer."""
    if masks.dtype == torch.bool:
        masks = masks.view(torch.uint8)
    _expect_layer(desc, masks=masks)
    if packed is None:
        packed = torch.empty(mglu_packed_mask_bytes(desc), dtype=torch.uint8, device=masks.device)
    _expect(packed, "packed", min_bytes=mglu_packed_mask_bytes(desc))
    _check(_lib.load().mglu_pack_masks(desc, _ptr(masks, "masks"), _ptr(packed, "packed"), _stream(masks)))
    return packed


def _workspace(desc, device, workspace):
    need = mglu_workspace_bytes(desc)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    return workspace, (workspace.numel() if workspace is not None else 0)


def mglu_forward(desc, x, W_packed, masks_packed, out=None, workspace=None):
    if out is None:
        out = torch.empty(desc.tokens, desc.d_ff, dtype=x.dtype, device=x.device)
    workspace, ws_bytes = _workspace(desc, x.device, workspace)
    _expect_layer(desc, x=x, out=out, W_packed=W_packed, masks_packed=masks_packed)
    _check(_lib.load().mglu_forward(desc, _ptr(x, "x"), _ptr(W_packed, "W_packed"),
                                    _ptr(masks_packed, "masks_packed"), _ptr(out, "out"),
                                    _ptr(workspace, "workspace"), ws_bytes, _stream(x)))
    return out


def _variant(gate, mask_use, route_weights):
    if gate == "swish" and mask_use == "both" and route_weights is None:
        return None, None
    if route_weights is not None and route_weights.dtype != torch.float32:
        raise ValueError("route_weights must be float32")
    v = _lib.MgluVariant(_lib.MGLU_GATE[gate], _lib.MGLU_MASK_USE[mask_use], _ptr(route_weights, "route_weights"))
    return v, ctypes.byref(v)


def mglu_forward_variant(desc, x, W_packed, masks_packed, gate="swish", mask_use="both", route_weights=None,
                         out=None, workspace=None):
    """mglu_forward with another gate function, a partial-mask ablation and/or per-token route weights."""
    if out is None:
        out = torch.empty(desc.tokens, desc.d_ff, dtype=x.dtype, device=x.device)
    workspace, ws_bytes = _workspace(desc, x.device, workspace)
    keep, ref = _variant(gate, mask_use, route_weights)
    _expect_layer(desc, x=x, out=out, W_packed=W_packed, masks_packed=masks_packed)
    _expect(route_weights, "route_weights", desc.tokens * desc.n_masks, torch.float32)
    _check(_lib.load().mglu_forward_variant(desc, ref, _ptr(x, "x"), _ptr(W_packed, "W_packed"),
                                            _ptr(masks_packed, "masks_packed"), _ptr(out, "out"),
                                            _ptr(workspace, "workspace"), ws_bytes, _stream(x)))
    return out


def mglu_packed_mask_bytes_planar(desc):
    return _lib.load().mglu_packed_mask_bytes_planar(desc)


def mglu_pack_masks_planar(desc, masks, packed=None):
    """masks uint8/bool as for mglu_pack_masks -> the planar packed buffer that mglu_forward_routed reads."""
    if masks.dtype == torch.bool:
        masks = masks.view(torch.uint8)
    _expect_layer(desc, masks=masks)
    if packed is None:
        packed = torch.empty(mglu_packed_mask_bytes_planar(desc), dtype=torch.uint8, device=masks.device)
    _expect(packed, "packed", min_bytes=mglu_packed_mask_bytes_planar(desc))
    _check(_lib.load().mglu_pack_masks_planar(desc, _ptr(masks, "masks"), _ptr(packed, "packed"), _stream(masks)))
    return packed


def mglu_forward_routed(desc, x, W_packed, masks_planar, route_weights, k, gate="swish", out=None):
    """The Top-K routed layer on the planar mask format: only the selected masks' planes are read."""
    if out is None:
        out = torch.empty(desc.tokens, desc.d_ff, dtype=x.dtype, device=x.device)
    _expect_layer(desc, x=x, out=out, W_packed=W_packed)
    _expect(masks_planar, "masks_planar", min_bytes=mglu_packed_mask_bytes_planar(desc))
    _expect(route_weights, "route_weights", desc.tokens * desc.n_masks, torch.float32)
    _check(_lib.load().mglu_forward_routed(desc, _ptr(x, "x"), _ptr(W_packed, "W_packed"),
                                           _ptr(masks_planar, "masks_planar"), _ptr(route_weights, "route_weights"),
                                           int(k), _lib.MGLU_GATE[gate], _ptr(out, "out"), _stream(x)))
    return out


def mglu_route_topk(desc, x, Wr, k, weights=None):
    """Top-K router: softmax over the k largest logits of x Wr per token, 0 elsewhere; fp32 [T, n_masks]."""
    if weights is None:
        weights = torch.empty(desc.tokens, desc.n_masks, dtype=torch.float32, device=x.device)
    _expect(x, "x", desc.tokens * desc.d_model, _TORCH_OF[desc.dtype])
    _expect(Wr, "Wr", desc.d_model * desc.n_masks, _TORCH_OF[desc.dtype])
    _expect(weights, "weights", desc.tokens * desc.n_masks, torch.float32)
    _check(_lib.load().mglu_route_topk(desc, _ptr(x, "x"), _ptr(Wr, "Wr"), int(k), _ptr(weights, "weights"),
                                       _stream(x)))
    return weights


def mglu_linear_forward(desc, a, W_packed, out=None, workspace=None):
    """out = a W; desc.d_model is the reduction length, desc.d_ff the output width."""
    if out is None:
        out = torch.empty(desc.tokens, desc.d_ff, dtype=a.dtype, device=a.device)
    workspace, ws_bytes = _workspace(desc, a.device, workspace)
    _expect_layer(desc, x=a, out=out, W_packed=W_packed)
    _check(_lib.load().mglu_linear_forward(desc, _ptr(a, "a"), _ptr(W_packed, "W_packed"), _ptr(out, "out"),
                                           _ptr(workspace, "workspace"), ws_bytes, _stream(a)))
    return out


def mglu_ffn_forward(desc, x, W_packed, masks_packed, Wo_packed, gate="swish", mask_use="both",
                     route_weights=None, hidden=None, y=None, workspace=None):
    """y = MGLU(x) Wo (two launches); returns (y, hidden)."""
    if hidden is None:
        hidden = torch.empty(desc.tokens, desc.d_ff, dtype=x.dtype, device=x.device)
    if y is None:
        y = torch.empty(desc.tokens, desc.d_model, dtype=x.dtype, device=x.device)
    workspace, ws_bytes = _workspace(desc, x.device, workspace)
    keep, ref = _variant(gate, mask_use, route_weights)
    _expect_layer(desc, x=x, out=hidden, W_packed=W_packed, masks_packed=masks_packed)
    _expect(y, "y", desc.tokens * desc.d_model, x.dtype)
    down = MgluDesc(desc.tokens, desc.d_ff, desc.d_model, 1, desc.dtype, desc.w_layout)
    _expect(Wo_packed, "Wo_packed", min_bytes=mglu_packed_weight_bytes(down))
    _expect(route_weights, "route_weights", desc.tokens * desc.n_masks, torch.float32)
    _check(_lib.load().mglu_ffn_forward(desc, ref, _ptr(x, "x"), _ptr(W_packed, "W_packed"),
                                        _ptr(masks_packed, "masks_packed"), _ptr(Wo_packed, "Wo_packed"),
                                        _ptr(hidden, "hidden"), _ptr(y, "y"), _ptr(workspace, "workspace"),
                                        ws_bytes, _stream(x)))
    return y, hidden


def mglu_forward_bool(desc, x, W, masks, out=None, workspace=None):
    if masks.dtype == torch.bool:
        masks = masks.view(torch.uint8)
    if out is None:
        out = torch.empty(desc.tokens, desc.d_ff, dtype=x.dtype, device=x.device)
    if workspace is None:
        workspace = torch.zeros(mglu_forward_bool_workspace_bytes(desc), dtype=torch.uint8, device=x.device)
    _expect_layer(desc, x=x, out=out, W=W, masks=masks)
    _check(_lib.load().mglu_forward_bool(desc, _ptr(x, "x"), _ptr(W, "W"), _ptr(masks, "masks"),
                                         _ptr(out, "out"), _ptr(workspace, "workspace"),
                                         workspace.numel(), _stream(x)))
    return out


def mglu_forward_bool_static(desc, x, W, masks, out):
    """mglu_forward_bool staged in the library's own static device array; `out` is the caller's (nothing is allocated)."""
    if masks.dtype == torch.bool:
        masks = masks.view(torch.uint8)
    _expect_layer(desc, x=x, out=out, W=W, masks=masks)
    _check(_lib.load().mglu_forward_bool_static(desc, _ptr(x, "x"), _ptr(W, "W"), _ptr(masks, "masks"),
                                                _ptr(out, "out"), _stream(x)))
    return out


def mglu_projections(desc, x, W_packed, masks_packed, workspace=None):
    """Returns (t [T,d], gate [n_masks,T,d], value [n_masks,T,d]) in fp32."""
    T, d, n = desc.tokens, desc.d_ff, desc.n_masks
    t = torch.empty(T, d, dtype=torch.float32, device=x.device)
    gate = torch.empty(n, T, d, dtype=torch.float32, device=x.device)
    value = torch.empty(n, T, d, dtype=torch.float32, device=x.device)
    workspace, ws_bytes = _workspace(desc, x.device, workspace)
    _expect_layer(desc, x=x, W_packed=W_packed, masks_packed=masks_packed)
    _check(_lib.load().mglu_projections(desc, _ptr(x, "x"), _ptr(W_packed, "W_packed"),
                                        _ptr(masks_packed, "masks_packed"), _ptr(t, "t"),
                                        _ptr(gate, "gate"), _ptr(value, "value"),
                                        _ptr(workspace, "workspace"), ws_bytes, _stream(x)))
    return t, gate, value


def swiglu_forward(desc, x, Wg_packed, Wv_packed, out=None, workspace=None):
    if out is None:
        out = torch.empty(desc.tokens, desc.d_ff, dtype=x.dtype, device=x.device)
    workspace, ws_bytes = _workspace(desc, x.device, workspace)
    _expect_layer(desc, x=x, out=out, W_packed=Wg_packed)
    _expect(Wv_packed, "Wv_packed", min_bytes=mglu_packed_weight_bytes(desc))
    _check(_lib.load().swiglu_forward(desc, _ptr(x, "x"), _ptr(Wg_packed, "Wg_packed"),
                                      _ptr(Wv_packed, "Wv_packed"), _ptr(out, "out"),
                                      _ptr(workspace, "workspace"), ws_bytes, _stream(x)))
    return out


def mglu_describe_plan(desc, call="forward", route_k=1):
    """Name of the kernel instantiation `call` would launch for this descriptor (host only, no GPU needed);
    route_k is the k of mglu_forward_routed and ignored by the other calls."""
    buf = ctypes.create_string_buffer(256)
    _check(_lib.load().mglu_describe_plan(desc, _lib.MGLU_CALL[call], int(route_k), buf, len(buf)))
    return buf.value.decode()


def mglu_stream_read(buf, sink):
    _check(_lib.load().mglu_stream_read(_ptr(buf, "buf"), buf.numel() * buf.element_size(),
                                        _ptr(sink, "sink"), _stream(buf)))
