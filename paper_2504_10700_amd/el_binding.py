"""ctypes binding of the per-order channel-mixing linear (include/el.h): same names as the C
ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C

from .binding import SC_F32, SC_F64, ScError, _check, _ptr, _stream, lib  # noqa: F401

EXPORTS = ("el_forward", "el_workspace_bytes", "el_backward", "el_sc_is_fused", "el_sc_workspace_bytes",
           "el_sc_backward_workspace_bytes", "el_sc_backward",
           "el_sc_forward")


class el_config(C.Structure):
    _fields_ = [("struct_size", C.c_int32), ("k_in", C.c_int32), ("k_out", C.c_int32), ("l_max", C.c_int32),
                ("dtype", C.c_int32), ("device", C.c_int32)]


def make_config(k_in: int, k_out: int, l_max: int, dtype: int = SC_F32, device: int = 0) -> el_config:
    cfg = el_config()
    cfg.struct_size = C.sizeof(el_config)
    cfg.k_in, cfg.k_out, cfg.l_max, cfg.dtype, cfg.device = k_in, k_out, l_max, dtype, device
    return cfg


_vp, _i64 = C.c_void_p, C.c_int64
lib.el_forward.argtypes = [C.POINTER(el_config), _i64, _vp, _vp, _vp, _vp]
lib.el_workspace_bytes.argtypes = [C.POINTER(el_config), _i64, C.POINTER(C.c_size_t)]
lib.el_backward.argtypes = [C.POINTER(el_config), _i64, _vp, _vp, _vp, _vp, _vp, _vp, C.c_size_t, _vp]
lib.el_sc_is_fused.argtypes = [_vp, C.c_int32]
lib.el_sc_workspace_bytes.argtypes = [_vp, C.c_int32, _i64, C.POINTER(C.c_size_t)]
lib.el_sc_forward.argtypes = [_vp, C.c_int32, _i64, _vp, _vp, _vp, _vp, _vp, _vp, C.c_size_t, _vp]
lib.el_sc_backward_workspace_bytes.argtypes = [_vp, C.c_int32, _i64, C.POINTER(C.c_size_t)]
lib.el_sc_backward.argtypes = [_vp, C.c_int32, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, C.c_size_t, _vp]
for _name in EXPORTS:
    getattr(lib, _name).restype = C.c_int


def el_forward(cfg: el_config, n_nodes: int, X, W, Y, stream=None) -> None:
    _check(lib.el_forward(C.byref(cfg), n_nodes, _ptr(X), _ptr(W), _ptr(Y), _stream(stream)))


def el_workspace_bytes(cfg: el_config, n_nodes: int) -> int:
    n = C.c_size_t()
    _check(lib.el_workspace_bytes(C.byref(cfg), n_nodes, C.byref(n)))
    return n.value


def el_backward(cfg: el_config, n_nodes: int, X, W, dY, dX, dW, workspace, workspace_bytes: int, stream=None) -> None:
    _check(lib.el_backward(C.byref(cfg), n_nodes, _ptr(X), _ptr(W), _ptr(dY), _ptr(dX), _ptr(dW), _ptr(workspace),
                           workspace_bytes, _stream(stream)))


def el_sc_is_fused(plan, k_in: int) -> bool:
    return bool(lib.el_sc_is_fused(plan.handle, k_in))


def el_sc_workspace_bytes(plan, k_in: int, n_nodes: int) -> int:
    n = C.c_size_t()
    _check(lib.el_sc_workspace_bytes(plan.handle, k_in, n_nodes, C.byref(n)))
    return n.value


def el_sc_forward(plan, k_in: int, n_nodes: int, X, W_lin, z, W, B, workspace, workspace_bytes: int,
                  stream=None) -> None:
    _check(lib.el_sc_forward(plan.handle, k_in, n_nodes, _ptr(X), _ptr(W_lin), _ptr(z), _ptr(W), _ptr(B), _ptr(workspace),
                             workspace_bytes, _stream(stream)))


def el_sc_backward_workspace_bytes(plan, k_in: int, n_nodes: int) -> int:
    n = C.c_size_t()
    _check(lib.el_sc_backward_workspace_bytes(plan.handle, k_in, n_nodes, C.byref(n)))
    return n.value


def el_sc_backward(plan, k_in: int, n_nodes: int, X, W_lin, z, W, dB, dX, dW_lin, dW, workspace, workspace_bytes: int,
                   stream=None) -> None:
    _check(lib.el_sc_backward(plan.handle, k_in, n_nodes, _ptr(X), _ptr(W_lin), _ptr(z), _ptr(W), _ptr(dB), _ptr(dX),
                              _ptr(dW_lin), _ptr(dW), _ptr(workspace), workspace_bytes, _stream(stream)))
