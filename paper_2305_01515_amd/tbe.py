"""Python binding of libtbe (include/tbe.h): argument marshalling only.

Every step of the path runs in the HIP kernels of the library; torch is used to
hold device memory and streams.  There is no fallback: if the library cannot be
loaded the import of this module's `lib()` fails.
"""
from __future__ import annotations

import collections
import ctypes as C
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtbe.so")

FP32, FP16 = 0, 1
ERRORS = {0: "TBE_OK", -1: "TBE_EINVAL", -2: "TBE_ERANGE", -3: "TBE_EORDER", -4: "TBE_ENOMEM", -5: "TBE_ELIMIT",
          -6: "TBE_EMISMATCH", -7: "TBE_EHIP"}
EXPORTS = ["tbe_create", "tbe_prefetch", "tbe_forward", "tbe_backward_update", "tbe_flush", "tbe_destroy",
           "tbe_get_stats", "tbe_num_sets", "tbe_export_cache_state", "tbe_export_batch_events", "tbe_last_error",
           "tbe_host_alloc", "tbe_host_free", "tbe_set_profiling", "tbe_get_stage_times", "tbe_set_inputs_ready",
           "tbe_set_policy", "tbe_export_cache_freq", "tbe_plan_placement", "tbe_set_pooling",
           "tbe_set_prefetch_queue", "tbe_set_prefetch_depth", "tbe_get_prefetch_depth", "tbe_set_backing_throttle", "tbe_set_probe_grouping", "tbe_enable_deferred_init", "tbe_export_initialised", "tbe_enable_second_level", "tbe_num_sets2", "tbe_export_second_level_state", "tbe_get_second_level_stats", "tbe_export_argmax", "tbe_backward_update_static", "tbe_import_cache_freq"]
POLICIES = {"lru": 0, "lfu": 1}
POOLINGS = {"sum": 0, "mean": 1, "max": 2}
STAGES = {"prefetch": 0, "fill": 1, "forward": 2, "backward_combine": 3, "backward_short": 4, "commit": 5, "backward_single": 6, "backward_heavy": 7, "backward": 8}


class TableSpec(C.Structure):
    _fields_ = [("rows", C.c_int64), ("dim", C.c_int32), ("dtype", C.c_int32), ("host_weights", C.c_void_p),
                ("host_state", C.c_void_p), ("cache_slots", C.c_int64)]


class BatchStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in
                ("lookups", "uniques", "hits", "inserts", "bypasses", "evictions", "hit_lookups")]

    def as_dict(self) -> Dict[str, int]:
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class Stats(C.Structure):
    _fields_ = [("last", BatchStats), ("total", BatchStats), ("h2d_bytes", C.c_int64), ("d2h_bytes", C.c_int64),
                ("late_fetches", C.c_int64), ("batch_id", C.c_int32), ("last_long_rows", C.c_int32)]


class TbeError(RuntimeError):
    def __init__(self, code: int, what: str, detail: str = ""):
        super().__init__(f"{what}: {ERRORS.get(code, code)} {detail}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """Load libtbe.so (building it first only when it does not exist)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build()
        l = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        l.tbe_create.argtypes = [C.POINTER(vp), C.POINTER(TableSpec), i32, i32, i32, i64, vp, vp]
        l.tbe_prefetch.argtypes = [vp, vp, vp, i32, i64]
        l.tbe_forward.argtypes = [vp, vp, vp, i32, i64, vp]
        l.tbe_backward_update.argtypes = [vp, vp, C.c_float, C.c_float]
        l.tbe_backward_update_static.argtypes = [vp, vp, C.c_float, C.c_float]
        l.tbe_flush.argtypes = [vp]
        l.tbe_destroy.argtypes = [vp]
        l.tbe_get_stats.argtypes = [vp, C.POINTER(Stats)]
        l.tbe_num_sets.argtypes = [vp, i32]
        l.tbe_num_sets.restype = i64
        l.tbe_export_cache_state.argtypes = [vp, i32, vp, vp]
        l.tbe_export_batch_events.argtypes = [vp, i32, i64, vp, vp, vp, vp]
        l.tbe_export_batch_events.restype = i64
        l.tbe_last_error.argtypes = [vp]
        l.tbe_last_error.restype = C.c_char_p
        l.tbe_host_alloc.argtypes = [C.POINTER(vp), C.c_size_t]
        l.tbe_host_free.argtypes = [vp]
        l.tbe_set_profiling.argtypes = [vp, i32]
        l.tbe_set_inputs_ready.argtypes = [vp, i32]
        l.tbe_set_policy.argtypes = [vp, i32]
        l.tbe_set_pooling.argtypes = [vp, i32]
        l.tbe_export_argmax.argtypes = [vp, vp]
        l.tbe_enable_second_level.argtypes = [vp, i32]
        l.tbe_set_prefetch_queue.argtypes = [vp, i32]
        l.tbe_set_prefetch_depth.argtypes = [vp, i32]
        l.tbe_get_prefetch_depth.argtypes = [vp, C.POINTER(i32), C.POINTER(i64)]
        l.tbe_set_backing_throttle.argtypes = [vp, i64]
        l.tbe_set_probe_grouping.argtypes = [vp, i32]
        l.tbe_enable_deferred_init.argtypes = [vp, C.c_uint64, C.c_float]
        l.tbe_export_initialised.argtypes = [vp, i32, vp]
        l.tbe_num_sets2.argtypes = [vp, i32]
        l.tbe_num_sets2.restype = i64
        l.tbe_export_second_level_state.argtypes = [vp, i32, vp, vp]
        l.tbe_get_second_level_stats.argtypes = [vp, vp, vp]
        l.tbe_export_cache_freq.argtypes = [vp, i32, vp]
        l.tbe_import_cache_freq.argtypes = [vp, i32, vp]
        l.tbe_get_stage_times.argtypes = [vp, i32, i64, vp]
        l.tbe_get_stage_times.restype = i64
        _lib = l
    return _lib


def pinned_empty(shape, dtype: torch.dtype) -> torch.Tensor:
    """A new pinned (device-visible) host tensor for the backing tier."""
    return torch.empty(shape, dtype=dtype, pin_memory=True)


class TBE:
    """One handle of the library.  weights[t]: pinned host tensor [rows, dim] fp32 or
    fp16; state[t]: pinned host float32 [rows].  Both are the backing tier and are
    read and written by the GPU."""

    def __init__(self, weights: Sequence[torch.Tensor], state: Sequence[torch.Tensor], cache_slots: Sequence[int],
                 ways: int, max_batch: int, max_lookups: int, overlap: bool = True, policy: str = "lru",
                 pooling: str = "sum", second_level_factor: int = 0, deferred_init=None):
        self._h = C.c_void_p()
        T = len(weights)
        self.T, self.ways = T, ways
        self.weights, self.state = list(weights), list(state)
        specs = (TableSpec * T)()
        self.dims: List[int] = []
        for t, (w, m) in enumerate(zip(weights, state)):
            if w.device.type != "cpu" or m.device.type != "cpu" or not w.is_pinned() or not m.is_pinned():
                raise ValueError("backing tier tensors must be pinned host tensors")
            if not (w.is_contiguous() and m.is_contiguous() and m.dtype == torch.float32):
                raise ValueError("backing tier tensors must be contiguous; state must be float32")
            dt = {torch.float32: FP32, torch.float16: FP16}[w.dtype]
            specs[t] = TableSpec(w.shape[0], w.shape[1], dt, w.data_ptr(), m.data_ptr(), int(cache_slots[t]))
            self.dims.append(int(w.shape[1]))
        self.sum_dim = sum(self.dims)
        self.compute_stream = torch.cuda.current_stream()
        self.aux_stream = torch.cuda.Stream() if overlap else self.compute_stream
        rc = lib().tbe_create(C.byref(self._h), specs, T, ways, max_batch, max_lookups,
                              C.c_void_p(self.compute_stream.cuda_stream), C.c_void_p(self.aux_stream.cuda_stream))
        if rc:
            raise TbeError(rc, "tbe_create", lib().tbe_last_error(None).decode())
        # Tensors the library still reads are kept alive per batch: a record is opened by prefetch() (or by a
        # forward() that prefetches itself), gets the output at forward() and the gradient at backward_update(),
        # and is dropped three trained batches later -- the library's batch buffers rotate over three, and every
        # kernel that reads a batch's tensors is ordered before the prefetch stage of the third batch after it.
        self._ahead: collections.deque = collections.deque()    # prefetched, not forwarded yet
        self._current: Optional[list] = None                    # forwarded, not updated yet
        self._trained: collections.deque = collections.deque(maxlen=3)
        self._depth = 1
        self._forwarded = (0, None)
        if policy != "lru":
            self._check(lib().tbe_set_policy(self._h, POLICIES[policy]), "tbe_set_policy")
        if pooling != "sum":
            self._check(lib().tbe_set_pooling(self._h, POOLINGS[pooling]), "tbe_set_pooling")
        if second_level_factor:
            self._check(lib().tbe_enable_second_level(self._h, second_level_factor), "tbe_enable_second_level")
        if deferred_init is not None:  # (seed, std)
            self._check(lib().tbe_enable_deferred_init(self._h, int(deferred_init[0]), float(deferred_init[1])),
                        "tbe_enable_deferred_init")

    def _check(self, rc: int, what: str):
        if rc:
            raise TbeError(rc, what, lib().tbe_last_error(self._h).decode())

    def close(self):
        if self._h:
            lib().tbe_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @staticmethod
    def _batch_of(offsets: torch.Tensor, T: int) -> int:
        return (offsets.numel() - 1) // T

    def prefetch(self, indices: torch.Tensor, offsets: torch.Tensor):
        assert indices.is_cuda and offsets.is_cuda and indices.dtype == torch.int64 and offsets.dtype == torch.int64
        self._check(lib().tbe_prefetch(self._h, indices.data_ptr(), offsets.data_ptr(),
                                       self._batch_of(offsets, self.T), indices.numel()), "tbe_prefetch")
        self._ahead.append([indices, offsets])

    def forward(self, indices: torch.Tensor, offsets: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        B = self._batch_of(offsets, self.T)
        if out is None:
            out = torch.empty(B, self.sum_dim, dtype=torch.float32, device=indices.device)
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.numel() == B * self.sum_dim
        self._check(lib().tbe_forward(self._h, indices.data_ptr(), offsets.data_ptr(), B, indices.numel(),
                                      out.data_ptr()), "tbe_forward")
        self._forwarded = (B, indices.device)
        rec = self._ahead.popleft() if self._ahead else [indices, offsets]  # none pending: it prefetched itself
        rec.append(out)
        self._current = rec
        return out

    def argmax(self, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """max pooling, between forward and backward_update: int32 [B, sum_dim], position inside its bag
        of the lookup that supplied each pooled element (-1: empty bag)"""
        B, device = self._forwarded
        if device is None:  # nothing has been forwarded: the library reports the order error
            out = out if out is not None else torch.empty(1, dtype=torch.int32, device="cuda")
        elif out is None:
            out = torch.empty(B, self.sum_dim, dtype=torch.int32, device=device)
        assert out.is_cuda and out.dtype == torch.int32 and out.is_contiguous() and out.numel() >= B * self.sum_dim
        self._check(lib().tbe_export_argmax(self._h, out.data_ptr()), "tbe_export_argmax")
        return out

    def backward_update(self, grad_out: torch.Tensor, lr: float, eps: float):
        assert grad_out.is_cuda and grad_out.dtype == torch.float32 and grad_out.is_contiguous()
        self._check(lib().tbe_backward_update(self._h, grad_out.data_ptr(), lr, eps), "tbe_backward_update")
        self._retire(grad_out)

    def backward_update_static(self, grad_out: torch.Tensor, lr: float, eps: float):
        """backward_update with its scratch buffer in the library's static device array: allocates nothing"""
        assert grad_out.is_cuda and grad_out.dtype == torch.float32 and grad_out.is_contiguous()
        self._check(lib().tbe_backward_update_static(self._h, grad_out.data_ptr(), lr, eps), "tbe_backward_update_static")
        self._retire(grad_out)

    def _retire(self, grad_out: torch.Tensor):
        rec, self._current = (self._current or []), None
        rec.append(grad_out)
        self._trained.append(rec)

    def flush(self):
        self._check(lib().tbe_flush(self._h), "tbe_flush")

    def stats(self) -> Dict[str, object]:
        s = Stats()
        self._check(lib().tbe_get_stats(self._h, C.byref(s)), "tbe_get_stats")
        return {"last": s.last.as_dict(), "total": s.total.as_dict(), "h2d_bytes": int(s.h2d_bytes),
                "d2h_bytes": int(s.d2h_bytes), "late_fetches": int(s.late_fetches), "last_long_rows": int(s.last_long_rows), "batch_id": int(s.batch_id)}

    def set_inputs_ready(self, ready: bool):
        """ready=True: index/offset tensors given to prefetch() are complete when it is called"""
        self._check(lib().tbe_set_inputs_ready(self._h, 1 if ready else 0), "tbe_set_inputs_ready")

    def set_profiling(self, enable):
        """False / True, or 2: whole-stage brackets only (none around the backward's single kernels)"""
        self._check(lib().tbe_set_profiling(self._h, int(enable)), "tbe_set_profiling")

    def stage_times(self, stage: str) -> np.ndarray:
        """milliseconds of every recorded bracket of a stage (see STAGES)"""
        sid = STAGES[stage]
        n = int(lib().tbe_get_stage_times(self._h, sid, 0, None))
        if n < 0:
            self._check(n, "tbe_get_stage_times")
        ms = np.empty(n, dtype=np.float32)
        got = int(lib().tbe_get_stage_times(self._h, sid, n, ms.ctypes.data))
        if got < 0:
            self._check(got, "tbe_get_stage_times")
        return ms

    def num_sets(self, t: int) -> int:
        return int(lib().tbe_num_sets(self._h, t))

    def cache_state(self, t: int) -> Tuple[np.ndarray, np.ndarray]:
        n = self.num_sets(t) * self.ways
        tags = np.empty(n, dtype=np.int64)
        ts = np.empty(n, dtype=np.int32)
        self._check(lib().tbe_export_cache_state(self._h, t, tags.ctypes.data, ts.ctypes.data), "tbe_export_cache_state")
        return tags, ts

    def second_level_state(self, t: int) -> Tuple[np.ndarray, np.ndarray]:
        n = int(lib().tbe_num_sets2(self._h, t)) * self.ways
        tags = np.empty(n, dtype=np.int64)
        ts = np.empty(n, dtype=np.int32)
        self._check(lib().tbe_export_second_level_state(self._h, t, tags.ctypes.data, ts.ctypes.data),
                    "tbe_export_second_level_state")
        return tags, ts

    def second_level_stats(self):
        last, total = np.zeros(4, dtype=np.int64), np.zeros(4, dtype=np.int64)
        self._check(lib().tbe_get_second_level_stats(self._h, last.ctypes.data, total.ctypes.data),
                    "tbe_get_second_level_stats")
        names = ("hits", "demotions", "evictions", "bypasses")
        return dict(zip(names, last.tolist())), dict(zip(names, total.tolist()))

    def initialised(self, t: int) -> np.ndarray:
        out = np.empty(self.weights[t].shape[0], dtype=np.uint8)
        self._check(lib().tbe_export_initialised(self._h, t, out.ctypes.data), "tbe_export_initialised")
        return out

    def set_prefetch_queue(self, length: int):
        self._check(lib().tbe_set_prefetch_queue(self._h, length), "tbe_set_prefetch_queue")
        self._depth = length  # tensors of queued batches are kept alive that much longer

    def set_prefetch_depth(self, depth: int):
        """pipeline `depth` batches deep (before the first batch): tbe_prefetch may run that many batches ahead"""
        self._check(lib().tbe_set_prefetch_depth(self._h, depth), "tbe_set_prefetch_depth")
        # the library's batch buffers then rotate over 2 depth + 1
        self._trained = collections.deque(self._trained, maxlen=max(3, 2 * depth + 1))

    def prefetch_depth(self):
        """(depth, rows taken from an earlier batch's overflow copies before a forward)"""
        d, n = C.c_int32(), C.c_int64()
        self._check(lib().tbe_get_prefetch_depth(self._h, C.byref(d), C.byref(n)), "tbe_get_prefetch_depth")
        return int(d.value), int(n.value)

    def set_backing_throttle(self, ns_per_row: int):
        self._check(lib().tbe_set_backing_throttle(self._h, ns_per_row), "tbe_set_backing_throttle")

    def set_probe_grouping(self, min_windows: int):
        self._check(lib().tbe_set_probe_grouping(self._h, min_windows), "tbe_set_probe_grouping")

    def cache_freq(self, t: int) -> np.ndarray:
        f = np.empty(self.num_sets(t) * self.ways, dtype=np.int32)
        self._check(lib().tbe_export_cache_freq(self._h, t, f.ctypes.data), "tbe_export_cache_freq")
        return f

    def set_cache_freq(self, t: int, freq: np.ndarray):
        f = np.ascontiguousarray(freq, dtype=np.int32)
        assert f.size == self.num_sets(t) * self.ways
        self._check(lib().tbe_import_cache_freq(self._h, t, f.ctypes.data), "tbe_import_cache_freq")

    def events(self, kind: str):
        """kind 'hit' / 'bypass': (table, row); 'insert': (table, row, slot, old)."""
        kid = {"hit": 0, "insert": 1, "bypass": 2}[kind]
        n = int(lib().tbe_export_batch_events(self._h, kid, 0, None, None, None, None))
        if n < 0:
            self._check(n, "tbe_export_batch_events")
        arrs = [np.empty(n, dtype=np.int64) for _ in range(4)]
        got = int(lib().tbe_export_batch_events(self._h, kid, n, *[a.ctypes.data for a in arrs]))
        if got < 0:
            self._check(got, "tbe_export_batch_events")
        return tuple(arrs) if kid == 1 else (arrs[0], arrs[1])
