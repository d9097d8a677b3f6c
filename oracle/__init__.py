"""ctypes front end of the CPU oracle (oracle/tbe_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  It marshals numpy arrays into the C functions
and holds no arithmetic of its own.  It never imports the HIP package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tbe_oracle.c")
_LIB = os.path.join(_HERE, "libtbe_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over tables)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Spec(C.Structure):
    _fields_ = [("rows", C.c_int64), ("dim", C.c_int32), ("dtype", C.c_int32), ("weights", C.c_void_p),
                ("state", C.c_void_p), ("cache_slots", C.c_int64)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in
                ("lookups", "uniques", "hits", "inserts", "bypasses", "evictions", "hit_lookups")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_create.restype = C.c_void_p
        _lib.orc_create.argtypes = [C.POINTER(_Spec), C.c_int32, C.c_int32]
        _lib.orc_destroy.argtypes = [C.c_void_p]
        _lib.orc_set_threads.argtypes = [C.c_void_p, C.c_int]
        _lib.orc_prefetch.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64]
        _lib.orc_forward.argtypes = [C.c_void_p, C.c_void_p]
        _lib.orc_backward_update.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_float]
        _lib.orc_flush.argtypes = [C.c_void_p]
        _lib.orc_num_sets.restype = C.c_int64
        _lib.orc_num_sets.argtypes = [C.c_void_p, C.c_int32]
        _lib.orc_batch_id.restype = C.c_int32
        _lib.orc_batch_id.argtypes = [C.c_void_p]
        _lib.orc_export_cache_state.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        _lib.orc_export_cache_freq.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        _lib.orc_import_cache_freq.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        _lib.orc_set_policy.argtypes = [C.c_void_p, C.c_int32]
        _lib.orc_set_pooling.argtypes = [C.c_void_p, C.c_int32]
        _lib.orc_set_second_level.argtypes = [C.c_void_p, C.c_void_p]
        _lib.orc_set_second_level_lock.argtypes = [C.c_void_p, C.c_int32]
        _lib.orc_set_prefetch_lock.argtypes = [C.c_void_p, C.c_int32]
        _lib.orc_enable_deferred_init.argtypes = [C.c_void_p, C.c_uint64, C.c_double]
        _lib.orc_export_initialised.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        _lib.orc_init_sum.restype = C.c_int32
        _lib.orc_init_sum.argtypes = [C.c_uint64, C.c_int32, C.c_int64, C.c_int32]
        _lib.orc_init_value.restype = C.c_float
        _lib.orc_init_value.argtypes = [C.c_uint64, C.c_float, C.c_int32, C.c_int64, C.c_int32]
        _lib.orc_num_sets2.restype = C.c_int64
        _lib.orc_num_sets2.argtypes = [C.c_void_p, C.c_int32]
        _lib.orc_export_second_level.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        _lib.orc_get_second_level_stats.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.orc_get_stats.argtypes = [C.c_void_p, C.POINTER(Stats), C.POINTER(Stats)]
        _lib.orc_events.restype = C.c_int64
        _lib.orc_events.argtypes = [C.c_void_p, C.c_int] + [C.c_void_p] * 4
        _lib.orc_export_argmax.argtypes = [C.c_void_p, C.c_void_p]
        _lib.orc_export_row_peak.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        _lib.orc_read_row.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p]
        _lib.orc_double_to_half.restype = C.c_uint16
        _lib.orc_double_to_half.argtypes = [C.c_double]
        _lib.orc_half_to_double.restype = C.c_double
        _lib.orc_half_to_double.argtypes = [C.c_uint16]
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"oracle {what} failed with code {code}")
        self.code = code


class Oracle:
    """weights[t]: numpy [rows, dim] float32 or float16, state[t]: numpy [rows]
    float32 -- the backing tier, modified in place (C-contiguous, kept alive here)."""

    def __init__(self, weights: Sequence[np.ndarray], state: Sequence[np.ndarray], cache_slots: Sequence[int],
                 ways: int, threads: int = 1, policy: str = "lru", pooling: str = "sum",
                 second_level_slots: Optional[Sequence[int]] = None, deferred_init=None, second_level_lock: int = 2,
                 prefetch_lock: int = 0):
        self.weights = list(weights)
        self.state = list(state)
        self.ways = ways
        T = len(self.weights)
        specs = (_Spec * T)()
        self.dims: List[int] = []
        for t, (w, m) in enumerate(zip(self.weights, self.state)):
            assert w.flags.c_contiguous and m.flags.c_contiguous and m.dtype == np.float32
            assert w.dtype in (np.float32, np.float16) and w.ndim == 2 and m.shape == (w.shape[0],)
            specs[t] = _Spec(w.shape[0], w.shape[1], 0 if w.dtype == np.float32 else 1, w.ctypes.data,
                             m.ctypes.data, int(cache_slots[t]))
            self.dims.append(w.shape[1])
        self.sum_dim = sum(self.dims)
        self.T = T
        self.h = lib().orc_create(specs, T, ways)
        if not self.h:
            raise OracleError(-1, "create")
        lib().orc_set_threads(self.h, threads)
        rc = lib().orc_set_policy(self.h, {"lru": 0, "lfu": 1}[policy])
        if rc:
            raise OracleError(rc, "set_policy")
        rc = lib().orc_set_pooling(self.h, {"sum": 0, "mean": 1, "max": 2}[pooling])
        if rc:
            raise OracleError(rc, "set_pooling")
        if prefetch_lock:  # batches before the current one whose ways are locked as well (Section 5.7 at that depth)
            rc = lib().orc_set_prefetch_lock(self.h, prefetch_lock)
            if rc:
                raise OracleError(rc, "set_prefetch_lock")
        if second_level_slots is not None:
            s2 = np.ascontiguousarray(second_level_slots, dtype=np.int64)
            assert s2.shape == (T,)
            if second_level_lock != 2:  # 1: only the current batch's entries are locked (the plain reading)
                rc = lib().orc_set_second_level_lock(self.h, second_level_lock)
                if rc:
                    raise OracleError(rc, "set_second_level_lock")
            rc = lib().orc_set_second_level(self.h, s2.ctypes.data)
            if rc:
                raise OracleError(rc, "set_second_level")
        if deferred_init is not None:  # (seed, std)
            rc = lib().orc_enable_deferred_init(self.h, int(deferred_init[0]), float(deferred_init[1]))
            if rc:
                raise OracleError(rc, "enable_deferred_init")
        self.B = 0

    def initialised(self, t: int) -> np.ndarray:
        out = np.empty(self.weights[t].shape[0], dtype=np.uint8)
        rc = lib().orc_export_initialised(self.h, t, out.ctypes.data)
        if rc:
            raise OracleError(rc, "export_initialised")
        return out

    def close(self):
        if self.h:
            lib().orc_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def prefetch(self, indices: np.ndarray, offsets: np.ndarray, batch: Optional[int] = None):
        indices = np.ascontiguousarray(indices, dtype=np.int64)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        B = (offsets.size - 1) // self.T if batch is None else batch
        rc = lib().orc_prefetch(self.h, indices.ctypes.data, offsets.ctypes.data, B, indices.size)
        if rc:
            raise OracleError(rc, "prefetch")
        self.B = B

    def forward(self) -> np.ndarray:
        out = np.empty((self.B, self.sum_dim), dtype=np.float32)
        rc = lib().orc_forward(self.h, out.ctypes.data)
        if rc:
            raise OracleError(rc, "forward")
        return out

    def argmax(self) -> np.ndarray:
        """max pooling, between forward and backward_update: [B, sum of dims] position inside its bag of
        the lookup that supplied each pooled element (-1: empty bag)"""
        a = np.empty((self.B, self.sum_dim), dtype=np.int32)
        rc = lib().orc_export_argmax(self.h, a.ctypes.data)
        if rc:
            raise OracleError(rc, "export_argmax")
        return a

    def backward_update(self, grad_out: np.ndarray, lr: float, eps: float):
        g = np.ascontiguousarray(grad_out, dtype=np.float32)
        assert g.shape == (self.B, self.sum_dim)
        rc = lib().orc_backward_update(self.h, g.ctypes.data, lr, eps)
        if rc:
            raise OracleError(rc, "backward_update")

    def flush(self):
        rc = lib().orc_flush(self.h)
        if rc:
            raise OracleError(rc, "flush")

    def num_sets(self, t: int) -> int:
        return int(lib().orc_num_sets(self.h, t))

    def batch_id(self) -> int:
        return int(lib().orc_batch_id(self.h))

    def cache_state(self, t: int):
        n = self.num_sets(t) * self.ways
        tags = np.empty(n, dtype=np.int64)
        ts = np.empty(n, dtype=np.int32)
        lib().orc_export_cache_state(self.h, t, tags.ctypes.data, ts.ctypes.data)
        return tags, ts

    def second_level_state(self, t: int):
        n = int(lib().orc_num_sets2(self.h, t)) * self.ways
        tags = np.empty(n, dtype=np.int64)
        ts = np.empty(n, dtype=np.int32)
        lib().orc_export_second_level(self.h, t, tags.ctypes.data, ts.ctypes.data)
        return tags, ts

    def second_level_stats(self):
        """(last batch, total), each {'hits', 'demotions', 'evictions', 'bypasses'}"""
        last, total = np.zeros(4, dtype=np.int64), np.zeros(4, dtype=np.int64)
        lib().orc_get_second_level_stats(self.h, last.ctypes.data, total.ctypes.data)
        names = ("hits", "demotions", "evictions", "bypasses")
        return dict(zip(names, last.tolist())), dict(zip(names, total.tolist()))

    def cache_freq(self, t: int) -> np.ndarray:
        f = np.empty(self.num_sets(t) * self.ways, dtype=np.int32)
        lib().orc_export_cache_freq(self.h, t, f.ctypes.data)
        return f

    def set_cache_freq(self, t: int, freq: np.ndarray):
        """test hook: overwrite the per-entry lookup counts of table t"""
        f = np.ascontiguousarray(freq, dtype=np.int32)
        assert f.size == self.num_sets(t) * self.ways
        rc = lib().orc_import_cache_freq(self.h, t, f.ctypes.data)
        if rc:
            raise OracleError(rc, "import_cache_freq")

    def stats(self):
        last, total = Stats(), Stats()
        lib().orc_get_stats(self.h, C.byref(last), C.byref(total))
        return last.as_dict(), total.as_dict()

    def events(self, kind: str):
        """kind 'hit' / 'bypass': (table, row); 'insert': (table, row, slot, old)."""
        kid = {"hit": 0, "insert": 1, "bypass": 2}[kind]
        n = int(lib().orc_events(self.h, kid, None, None, None, None))
        arrs = [np.empty(n, dtype=np.int64) for _ in range(4)]
        lib().orc_events(self.h, kid, *[a.ctypes.data for a in arrs])
        return tuple(arrs) if kid == 1 else (arrs[0], arrs[1])

    def row_peak(self, t: int) -> np.ndarray:
        """float32 [rows]: the largest |element| each row has held before or after any of its updates (0: never
        updated).  Bookkeeping for the tests' error bars; it enters no result."""
        p = np.empty(self.weights[t].shape[0], dtype=np.float32)
        rc = lib().orc_export_row_peak(self.h, t, p.ctypes.data)
        if rc:
            raise OracleError(rc, "export_row_peak")
        return p

    def read_row(self, t: int, r: int):
        w = np.empty(self.dims[t], dtype=np.float64)
        m = C.c_float()
        rc = lib().orc_read_row(self.h, t, r, w.ctypes.data, C.byref(m))
        if rc:
            raise OracleError(rc, "read_row")
        return w, float(m.value)
