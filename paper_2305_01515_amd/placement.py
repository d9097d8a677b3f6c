"""Binding of the table-assignment solver of libtbe (tbe_plan_placement; paper Section
5.6.1, Eq. 6) and the helper that turns an assignment into per-table cache sizes.
Argument marshalling only: the search runs in the library."""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence, Tuple

from . import tbe as _tbe


class PlaceTable(C.Structure):
    _fields_ = [("bytes", C.c_int64), ("traffic", C.c_double)]


class PlaceMemory(C.Structure):
    _fields_ = [("capacity_bytes", C.c_int64), ("bandwidth", C.c_double)]


def _solver_library():
    """the library that exports tbe_plan_placement (libtbe; the sanitizer run of the tests swaps in a host-only build)"""
    return _tbe.lib()


def plan(size: Sequence[int], traffic: Sequence[float], capacity: Sequence[int], bandwidth: Sequence[float],
         max_nodes: int = 0) -> Optional[Tuple[List[int], float, bool]]:
    """(memory type of every table, lookup time of Eq. 6, proven optimal) or None when no
    assignment fits."""
    T, M = len(size), len(capacity)
    if len(traffic) != T or len(bandwidth) != M:
        raise ValueError("size/traffic and capacity/bandwidth must have equal lengths")
    l = _solver_library()
    l.tbe_plan_placement.argtypes = [C.POINTER(PlaceTable), C.c_int32, C.POINTER(PlaceMemory), C.c_int32, C.c_int64,
                                     C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_int32)]
    tabs = (PlaceTable * max(T, 1))(*[PlaceTable(int(s), float(x)) for s, x in zip(size, traffic)])
    mems = (PlaceMemory * max(M, 1))(*[PlaceMemory(int(c), float(b)) for c, b in zip(capacity, bandwidth)])
    out = (C.c_int32 * max(T, 1))()
    t, opt = C.c_double(), C.c_int32()
    rc = l.tbe_plan_placement(tabs, T, mems, M, max_nodes, out, C.byref(t), C.byref(opt))
    if rc == -5:  # TBE_ELIMIT: nothing fits
        return None
    if rc:
        raise ValueError(f"tbe_plan_placement: {_tbe.ERRORS.get(rc, rc)}")
    return list(out[:T]), float(t.value), bool(opt.value)
