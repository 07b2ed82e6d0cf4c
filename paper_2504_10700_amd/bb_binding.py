"""ctypes binding of the load balancer (include/bb.h): same name as the C ABI, argument
marshalling only.  Host arrays are numpy int32."""
from __future__ import annotations

import ctypes as C
from typing import Tuple

import numpy as np

from .binding import ScError, _check, lib  # noqa: F401

EXPORTS = ("bb_create_balanced_batches",)

lib.bb_create_balanced_batches.argtypes = [C.POINTER(C.c_int32), C.c_int64, C.c_int64, C.c_int32,
                                           C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int64)]
lib.bb_create_balanced_batches.restype = C.c_int


def bb_create_balanced_batches(sizes, capacity: int, n_gpus: int) -> Tuple[np.ndarray, np.ndarray, int]:
    """Returns (bin_of_graph, slot_of_graph, n_bins)."""
    sizes = np.ascontiguousarray(sizes, dtype=np.int32)
    n = int(sizes.size)
    bins = np.full(n, -1, dtype=np.int32)
    slots = np.full(n, -1, dtype=np.int32)
    n_bins = C.c_int64()
    ip = C.POINTER(C.c_int32)
    _check(lib.bb_create_balanced_batches(sizes.ctypes.data_as(ip), n, int(capacity), int(n_gpus),
                                          bins.ctypes.data_as(ip), slots.ctypes.data_as(ip), C.byref(n_bins)))
    return bins, slots, n_bins.value
