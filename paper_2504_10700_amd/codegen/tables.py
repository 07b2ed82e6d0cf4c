"""Access to the library's own coupling tables for the kernel generator.

The generator never derives Clebsch-Gordan data itself: the real-basis coupling
tensors, the external path list and the sparse polynomial of every external path
come from the C-ABI library's host-side table builder (sc_coupling_tensor,
sc_plan_paths, sc_plan_path_terms on a host-only plan).  Needs no GPU.
"""
from __future__ import annotations

import ctypes as C
import functools
import os
from typing import List, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
HOST_LIB = os.path.join(os.path.dirname(_HERE), "libsc_mi355x.so")

SC_MAX_OUT = 4


class _Config(C.Structure):
    _fields_ = [("struct_size", C.c_int32), ("num_channels", C.c_int32), ("l_max", C.c_int32),
                ("nu_max", C.c_int32), ("num_elements", C.c_int32), ("num_out", C.c_int32),
                ("out_l", C.c_int32 * SC_MAX_OUT), ("out_parity", C.c_int32 * SC_MAX_OUT),
                ("dtype", C.c_int32), ("device", C.c_int32), ("flags", C.c_uint32), ("tile_nodes", C.c_int32)]


class Tables:
    def __init__(self, lib_path: str, l_max: int, nu_max: int, outs: Sequence[Tuple[int, int]]):
        self.lib = C.CDLL(lib_path)
        self.lib.sc_last_error.restype = C.c_char_p
        self.l_max, self.nu_max, self.outs = l_max, nu_max, list(outs)
        cfg = _Config()
        cfg.struct_size = C.sizeof(_Config)
        cfg.num_channels, cfg.l_max, cfg.nu_max, cfg.num_elements = 64, l_max, nu_max, 1
        cfg.num_out = len(outs)
        for i, (L, p) in enumerate(outs):
            cfg.out_l[i], cfg.out_parity[i] = L, p
        cfg.dtype, cfg.device, cfg.flags = 1, 0, 1 | 2      # f64, host only, generic
        self.plan = C.c_void_p()
        self._check(self.lib.sc_plan_create(C.byref(cfg), C.byref(self.plan)))
        info = (C.c_int32 * 10)()   # sc_info: four counts, then ops[3] and flops[3]
        self._check(self.lib.sc_plan_info(self.plan, info))
        self.n_lm, self.n_LM, self.num_paths = info[0], info[1], info[2]
        paths = np.zeros((self.num_paths, 6), dtype=np.int32)
        self._check(self.lib.sc_plan_paths(self.plan, paths.ctypes.data_as(C.POINTER(C.c_int32))))
        self.paths = [tuple(int(x) for x in r) for r in paths]

    def _check(self, st):
        if st != 0:
            raise RuntimeError(self.lib.sc_last_error().decode())

    @functools.lru_cache(maxsize=None)
    def cg(self, l1: int, l2: int, l3: int) -> np.ndarray:
        out = np.zeros((2 * l1 + 1, 2 * l2 + 1, 2 * l3 + 1))
        self._check(self.lib.sc_coupling_tensor(l1, l2, l3, out.ctypes.data_as(C.POINTER(C.c_double))))
        out.setflags(write=False)
        return out

    def path_terms(self, p: int):
        n = C.c_int32()
        self._check(self.lib.sc_plan_path_terms(self.plan, p, 0, C.byref(n), None, None, None, None, None))
        M, i1, i2, i3 = (np.zeros(max(n.value, 1), dtype=np.int32) for _ in range(4))
        coef = np.zeros(max(n.value, 1))
        if n.value:
            ip = C.POINTER(C.c_int32)
            self._check(self.lib.sc_plan_path_terms(self.plan, p, n.value, C.byref(n), M.ctypes.data_as(ip),
                                                    i1.ctypes.data_as(ip), i2.ctypes.data_as(ip),
                                                    i3.ctypes.data_as(ip), coef.ctypes.data_as(C.POINTER(C.c_double))))
        k = n.value
        return M[:k], i1[:k], i2[:k], i3[:k], coef[:k]

    def eval_external(self, p: int, a: np.ndarray) -> np.ndarray:
        """P_{p,M}(a) for samples a[n, n_lm] -> [n, 2L+1] from the library's sparse terms."""
        nu, out = self.paths[p][0], self.paths[p][1]
        L = self.outs[out][0]
        res = np.zeros((a.shape[0], 2 * L + 1))
        M, i1, i2, i3, coef = self.path_terms(p)
        for t in range(len(M)):
            v = coef[t] * a[:, i1[t]]
            if nu >= 2:
                v = v * a[:, i2[t]]
            if nu >= 3:
                v = v * a[:, i3[t]]
            res[:, M[t]] += v
        return res
