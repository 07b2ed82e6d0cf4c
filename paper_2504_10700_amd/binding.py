"""Thin ctypes binding of libsc_mi355x.so (the C ABI declared in include/sc.h).

Argument marshalling only: every step of the contraction runs in the library's
HIP kernels.  Tensor arguments may be torch tensors living on the GPU (their
data_ptr() is passed) or raw integer device addresses.  There is no CPU
fallback: if the library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np
# torch ships its own HIP runtime (same soname as the system one).  It has to be
# loaded first so that this library binds to that copy and both share one runtime:
# device pointers and streams cross the boundary.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SC_LIB_PATH", os.path.join(_HERE, "libsc_mi355x.so"))  # override: development only

SC_OK = 0
SC_ERR_INVALID_ARG, SC_ERR_UNSUPPORTED, SC_ERR_WORKSPACE, SC_ERR_HIP, SC_ERR_ALLOC = 1, 2, 3, 4, 5
SC_F32, SC_F64, SC_BF16 = 0, 1, 2
SC_MAX_OUT = 4
SC_PLAN_HOST_ONLY, SC_PLAN_FORCE_GENERIC, SC_PLAN_WINDOW_ORDER = 1, 2, 4
SC_REUSE_GROUPING, SC_REUSE_WEIGHTS, SC_Z_GROUPED, SC_COMPONENT_MAJOR = 1, 2, 4, 8
SC_NOALLOC_MAX_NODES, SC_NOALLOC_SCRATCH_BYTES = 65536, 8 << 20

EXPORTS = ("sc_plan_create", "sc_plan_destroy", "sc_plan_info", "sc_plan_paths", "sc_plan_path_terms",
           "sc_coupling_tensor", "sc_workspace_bytes", "sc_forward", "sc_forward_noalloc", "sc_backward",
           "sc_double_backward",
           "sc_profile_enable", "sc_profile_read", "sc_profile_read_double_backward", "sc_probe_stream",
           "sc_last_error")


class sc_config(C.Structure):
    _fields_ = [("struct_size", C.c_int32), ("num_channels", C.c_int32), ("l_max", C.c_int32),
                ("nu_max", C.c_int32), ("num_elements", C.c_int32), ("num_out", C.c_int32),
                ("out_l", C.c_int32 * SC_MAX_OUT), ("out_parity", C.c_int32 * SC_MAX_OUT),
                ("dtype", C.c_int32), ("device", C.c_int32), ("flags", C.c_uint32), ("tile_nodes", C.c_int32)]


class sc_info(C.Structure):
    _fields_ = [("n_lm", C.c_int32), ("n_LM", C.c_int32), ("num_paths", C.c_int32), ("specialised", C.c_int32),
                ("ops", C.c_int32 * 3), ("flops", C.c_int32 * 3)]


class ScError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"sc status {status}: {message}")
        self.status = status


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is not built. Run `python -c 'import __graft_entry__ as g; g.build()'` at the repo root; "
            "there is no fallback path.")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, u32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32
    lib.sc_plan_create.argtypes = [C.POINTER(sc_config), C.POINTER(vp)]
    lib.sc_plan_destroy.argtypes = [vp]
    lib.sc_plan_info.argtypes = [vp, C.POINTER(sc_info)]
    lib.sc_plan_paths.argtypes = [vp, C.POINTER(i32)]
    lib.sc_plan_path_terms.argtypes = [vp, i32, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32),
                                       C.POINTER(i32), C.POINTER(i32), C.POINTER(C.c_double)]
    lib.sc_coupling_tensor.argtypes = [i32, i32, i32, C.POINTER(C.c_double)]
    lib.sc_workspace_bytes.argtypes = [vp, i64, C.POINTER(C.c_size_t)]
    lib.sc_forward.argtypes = [vp, i64, vp, vp, vp, vp, vp, C.c_size_t, u32, vp]
    lib.sc_forward_noalloc.argtypes = [vp, i64, vp, vp, vp, vp, vp]
    lib.sc_backward.argtypes = [vp, i64, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, u32, vp]
    lib.sc_double_backward.argtypes = [vp, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, u32, vp]
    lib.sc_probe_stream.argtypes = [i32, vp, vp, vp, vp, i64, vp]
    lib.sc_profile_enable.argtypes = [vp, i32]
    lib.sc_profile_read_double_backward.argtypes = [vp, C.POINTER(C.c_float)]
    lib.sc_profile_read.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_float)]
    lib.sc_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if name != "sc_last_error":
            getattr(lib, name).restype = C.c_int
    return lib


lib = _load()


def _check(status: int) -> None:
    if status != SC_OK:
        raise ScError(status, sc_last_error())


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()  # torch tensor


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


class Plan:
    """Owner of an sc_plan*; freed by sc_plan_destroy or on garbage collection."""

    def __init__(self, handle: int, cfg: sc_config):
        self.handle = handle
        self.cfg = cfg

    def __del__(self):
        try:
            sc_plan_destroy(self)
        except Exception:
            pass


def sc_last_error() -> str:
    return lib.sc_last_error().decode()


def sc_plan_create(num_channels: int, l_max: int, nu_max: int, num_elements: int,
                   out_irreps: Sequence[Tuple[int, int]], dtype: int = SC_F32, device: int = 0,
                   flags: int = 0, tile_nodes: int = 0) -> Plan:
    cfg = sc_config()
    cfg.struct_size = C.sizeof(sc_config)
    cfg.num_channels, cfg.l_max, cfg.nu_max, cfg.num_elements = num_channels, l_max, nu_max, num_elements
    cfg.num_out = len(out_irreps)
    for i, (L, p) in enumerate(out_irreps[:SC_MAX_OUT]):
        cfg.out_l[i], cfg.out_parity[i] = L, p
    cfg.dtype, cfg.device, cfg.flags, cfg.tile_nodes = dtype, device, flags, tile_nodes
    h = C.c_void_p()
    _check(lib.sc_plan_create(C.byref(cfg), C.byref(h)))
    return Plan(h.value, cfg)


def sc_plan_destroy(plan: Optional[Plan]) -> None:
    if plan is None or plan.handle is None:
        return
    h, plan.handle = plan.handle, None
    _check(lib.sc_plan_destroy(h))


def sc_plan_info(plan: Plan) -> sc_info:
    info = sc_info()
    _check(lib.sc_plan_info(plan.handle, C.byref(info)))
    return info


def sc_plan_paths(plan: Plan) -> np.ndarray:
    P = sc_plan_info(plan).num_paths
    out = np.zeros((P, 6), dtype=np.int32)
    _check(lib.sc_plan_paths(plan.handle, out.ctypes.data_as(C.POINTER(C.c_int32))))
    return out


def sc_plan_path_terms(plan: Plan, path: int):
    """(M, i1, i2, i3, coef) arrays of one path's sparse terms."""
    n = C.c_int32()
    _check(lib.sc_plan_path_terms(plan.handle, path, 0, C.byref(n), None, None, None, None, None))
    M, i1, i2, i3 = (np.zeros(n.value, dtype=np.int32) for _ in range(4))
    coef = np.zeros(n.value, dtype=np.float64)
    if n.value:
        ip = C.POINTER(C.c_int32)
        _check(lib.sc_plan_path_terms(plan.handle, path, n.value, C.byref(n), M.ctypes.data_as(ip),
                                      i1.ctypes.data_as(ip), i2.ctypes.data_as(ip), i3.ctypes.data_as(ip),
                                      coef.ctypes.data_as(C.POINTER(C.c_double))))
    return M, i1, i2, i3, coef


def sc_coupling_tensor(l1: int, l2: int, l3: int) -> np.ndarray:
    out = np.zeros((2 * l1 + 1, 2 * l2 + 1, 2 * l3 + 1), dtype=np.float64)
    _check(lib.sc_coupling_tensor(l1, l2, l3, out.ctypes.data_as(C.POINTER(C.c_double))))
    return out


def sc_workspace_bytes(plan: Plan, n_nodes: int) -> int:
    b = C.c_size_t()
    _check(lib.sc_workspace_bytes(plan.handle, n_nodes, C.byref(b)))
    return b.value


def sc_forward(plan: Plan, n_nodes: int, A, z, W, B, workspace, workspace_bytes: int, flags: int = 0,
               stream=None) -> None:
    _check(lib.sc_forward(plan.handle, n_nodes, _ptr(A), _ptr(z), _ptr(W), _ptr(B), _ptr(workspace),
                          workspace_bytes, flags, _stream(stream)))


def sc_forward_noalloc(plan: Plan, n_nodes: int, A, z, W, B, stream=None) -> None:
    _check(lib.sc_forward_noalloc(plan.handle, n_nodes, _ptr(A), _ptr(z), _ptr(W), _ptr(B), _stream(stream)))


def sc_backward(plan: Plan, n_nodes: int, A, z, W, dB, dA, dW, workspace, workspace_bytes: int, flags: int = 0,
                stream=None) -> None:
    _check(lib.sc_backward(plan.handle, n_nodes, _ptr(A), _ptr(z), _ptr(W), _ptr(dB), _ptr(dA), _ptr(dW),
                           _ptr(workspace), workspace_bytes, flags, _stream(stream)))


def sc_double_backward(plan: Plan, n_nodes: int, A, z, W, dB, H, ddB, dA2, dW2, workspace, workspace_bytes: int,
                       flags: int = 0, stream=None) -> None:
    _check(lib.sc_double_backward(plan.handle, n_nodes, _ptr(A), _ptr(z), _ptr(W), _ptr(dB), _ptr(H), _ptr(ddB),
                                  _ptr(dA2), _ptr(dW2), _ptr(workspace), workspace_bytes, flags, _stream(stream)))


SC_PROBE_READ, SC_PROBE_WRITE, SC_PROBE_COPY, SC_PROBE_ROWS, SC_PROBE_ROWS_FORWARD = 0, 1, 2, 3, 4


def sc_probe_stream(kind: int, src, src2, dst, perm, n: int, stream=None) -> None:
    _check(lib.sc_probe_stream(kind, _ptr(src), _ptr(src2), _ptr(dst), _ptr(perm), n, _stream(stream)))


def sc_profile_enable(plan: Plan, on: bool) -> None:
    _check(lib.sc_profile_enable(plan.handle, 1 if on else 0))


def sc_profile_read(plan: Plan) -> Tuple[float, float]:
    """(forward_ms, backward_ms) of the main kernels of the latest bracketed calls."""
    f, b = C.c_float(), C.c_float()
    _check(lib.sc_profile_read(plan.handle, C.byref(f), C.byref(b)))
    return f.value, b.value


def sc_profile_read_double_backward(plan: Plan) -> float:
    """Duration in ms of the main kernel of the latest bracketed sc_double_backward call."""
    t = C.c_float()
    _check(lib.sc_profile_read_double_backward(plan.handle, C.byref(t)))
    return t.value
