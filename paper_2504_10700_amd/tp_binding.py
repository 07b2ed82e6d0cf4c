"""ctypes binding of the channelwise tensor product (include/tp.h): same names as the C ABI,
argument marshalling only.  Shares the loaded library, status codes and error handling with
binding.py."""
from __future__ import annotations

import ctypes as C
from typing import Tuple

import numpy as np

from . import binding as _b
from .binding import SC_F32, SC_F64, SC_PLAN_FORCE_GENERIC, SC_PLAN_HOST_ONLY, ScError, _check, _ptr, _stream, lib  # noqa: F401

EXPORTS = ("tp_plan_create", "tp_plan_destroy", "tp_plan_info", "tp_plan_paths", "tp_plan_terms", "tp_forward",
           "tp_workspace_bytes", "tp_backward", "tp_double_backward", "tp_profile_enable", "tp_profile_read",
           "tp_profile_read_double_backward")


class tp_config(C.Structure):
    _fields_ = [("struct_size", C.c_int32), ("num_channels", C.c_int32), ("l_Y", C.c_int32), ("l_h", C.c_int32),
                ("L_max", C.c_int32), ("dtype", C.c_int32), ("device", C.c_int32), ("flags", C.c_uint32)]


class tp_info(C.Structure):
    _fields_ = [("n_Y", C.c_int32), ("n_h", C.c_int32), ("n_out", C.c_int32), ("num_paths", C.c_int32),
                ("specialised", C.c_int32), ("ops", C.c_int32 * 3), ("flops", C.c_int32 * 3)]


def _declare() -> None:
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    pi32 = C.POINTER(i32)
    lib.tp_plan_create.argtypes = [C.POINTER(tp_config), C.POINTER(vp)]
    lib.tp_plan_destroy.argtypes = [vp]
    lib.tp_plan_info.argtypes = [vp, C.POINTER(tp_info)]
    lib.tp_plan_paths.argtypes = [vp, pi32]
    lib.tp_plan_terms.argtypes = [vp, i32, pi32, pi32, pi32, pi32, pi32, C.POINTER(C.c_double)]
    lib.tp_forward.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp]
    lib.tp_workspace_bytes.argtypes = [vp, i64, C.POINTER(C.c_size_t)]
    lib.tp_backward.argtypes = [vp, i64, i64, i64] + [vp] * 12 + [C.c_size_t, vp]
    lib.tp_double_backward.argtypes = [vp, i64, i64, i64] + [vp] * 16 + [C.c_size_t, vp]
    lib.tp_profile_read_double_backward.argtypes = [vp, C.POINTER(C.c_float)]
    lib.tp_profile_enable.argtypes = [vp, i32]
    lib.tp_profile_read.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_float)]
    for name in EXPORTS:
        getattr(lib, name).restype = C.c_int


_declare()


class Plan:
    """Owner of a tp_plan*; freed by tp_plan_destroy or on garbage collection."""

    def __init__(self, handle: int, cfg: tp_config):
        self.handle = handle
        self.cfg = cfg

    def __del__(self):
        try:
            tp_plan_destroy(self)
        except Exception:
            pass


def tp_plan_create(num_channels: int, l_Y: int, l_h: int, L_max: int, dtype: int = SC_F32, device: int = 0,
                   flags: int = 0) -> Plan:
    cfg = tp_config()
    cfg.struct_size = C.sizeof(tp_config)
    cfg.num_channels, cfg.l_Y, cfg.l_h, cfg.L_max = num_channels, l_Y, l_h, L_max
    cfg.dtype, cfg.device, cfg.flags = dtype, device, flags
    h = C.c_void_p()
    _check(lib.tp_plan_create(C.byref(cfg), C.byref(h)))
    return Plan(h.value, cfg)


def tp_plan_destroy(plan: Plan) -> None:
    if plan.handle:
        handle, plan.handle = plan.handle, None
        _check(lib.tp_plan_destroy(handle))


def tp_plan_info(plan: Plan) -> tp_info:
    info = tp_info()
    _check(lib.tp_plan_info(plan.handle, C.byref(info)))
    return info


def tp_plan_paths(plan: Plan) -> np.ndarray:
    """[num_paths, 3] rows (l1, l2, l3)."""
    P = tp_plan_info(plan).num_paths
    out = np.zeros((P, 3), dtype=np.int32)
    _check(lib.tp_plan_paths(plan.handle, out.ctypes.data_as(C.POINTER(C.c_int32))))
    return out


def tp_plan_terms(plan: Plan):
    """(path, a, b, c, coef) arrays of the non-zero coupling terms."""
    n = C.c_int32()
    _check(lib.tp_plan_terms(plan.handle, 0, C.byref(n), None, None, None, None, None))
    arrs = [np.zeros(n.value, dtype=np.int32) for _ in range(4)]
    coef = np.zeros(n.value, dtype=np.float64)
    _check(lib.tp_plan_terms(plan.handle, n.value, C.byref(n), *[x.ctypes.data_as(C.POINTER(C.c_int32)) for x in arrs],
                             coef.ctypes.data_as(C.POINTER(C.c_double))))
    return (*arrs, coef)


def tp_forward(plan: Plan, n_nodes_in: int, n_nodes_out: int, n_edges: int, Y, h, R, sender, row_ptr, A,
               stream=None) -> None:
    _check(lib.tp_forward(plan.handle, n_nodes_in, n_nodes_out, n_edges, _ptr(Y), _ptr(h), _ptr(R), _ptr(sender),
                          _ptr(row_ptr), _ptr(A), _stream(stream)))


def tp_workspace_bytes(plan: Plan, n_edges: int) -> int:
    n = C.c_size_t()
    _check(lib.tp_workspace_bytes(plan.handle, n_edges, C.byref(n)))
    return n.value


def tp_backward(plan: Plan, n_nodes_in: int, n_nodes_out: int, n_edges: int, Y, h, R, sender, row_ptr, send_ptr,
                send_edge, dA, dY, dh, dR, workspace, workspace_bytes: int, stream=None) -> None:
    _check(lib.tp_backward(plan.handle, n_nodes_in, n_nodes_out, n_edges, _ptr(Y), _ptr(h), _ptr(R), _ptr(sender),
                           _ptr(row_ptr), _ptr(send_ptr), _ptr(send_edge), _ptr(dA), _ptr(dY), _ptr(dh), _ptr(dR),
                           _ptr(workspace), workspace_bytes, _stream(stream)))


def tp_double_backward(plan: Plan, n_nodes_in: int, n_nodes_out: int, n_edges: int, Y, h, R, sender, row_ptr,
                       send_ptr, send_edge, dA, HY, Hh, HR, ddA, d2Y, d2h, d2R, workspace, workspace_bytes: int,
                       stream=None) -> None:
    _check(lib.tp_double_backward(plan.handle, n_nodes_in, n_nodes_out, n_edges, _ptr(Y), _ptr(h), _ptr(R),
                                  _ptr(sender), _ptr(row_ptr), _ptr(send_ptr), _ptr(send_edge), _ptr(dA), _ptr(HY),
                                  _ptr(Hh), _ptr(HR), _ptr(ddA), _ptr(d2Y), _ptr(d2h), _ptr(d2R), _ptr(workspace),
                                  workspace_bytes, _stream(stream)))


def tp_profile_read_double_backward(plan: Plan) -> float:
    t = C.c_float()
    _check(lib.tp_profile_read_double_backward(plan.handle, C.byref(t)))
    return t.value


def tp_profile_enable(plan: Plan, on: bool) -> None:
    _check(lib.tp_profile_enable(plan.handle, 1 if on else 0))


def tp_profile_read(plan: Plan) -> Tuple[float, float, float]:
    """(forward, edge-walking backward, per-sender dh sum) kernel durations in ms."""
    f, r, s = C.c_float(), C.c_float(), C.c_float()
    _check(lib.tp_profile_read(plan.handle, C.byref(f), C.byref(r), C.byref(s)))
    return f.value, r.value, s.value
