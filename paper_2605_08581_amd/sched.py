"""ctypes binding of the host control plane in libprism.so (argument marshalling
only): the query-aware scheduler and the demand-aware radix tree declared in
``include/prism_sched.h``.  Nothing here touches a device."""
from __future__ import annotations

import ctypes
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import binding as B

QAS_MODE_QAS, QAS_MODE_FIFO = 0, 1
EVICT_DART, EVICT_LRU, EVICT_LRU_ACTIVE, EVICT_LFU = 0, 1, 2, 3
POLICIES = {"dart": EVICT_DART, "lru": EVICT_LRU, "lru_active": EVICT_LRU_ACTIVE, "lfu": EVICT_LFU}
SPAN_NONE, SPAN_SYSTEM, SPAN_REUSABLE, SPAN_PRIVATE = -1, 0, 1, 2

EXPORTS = (
    "prism_qas_create", "prism_qas_destroy", "prism_qas_submit", "prism_qas_complete", "prism_qas_round",
    "prism_qas_round_hints", "prism_qas_round_segments", "prism_qas_round_priorities", "prism_qas_pending",
    "prism_qas_active", "prism_dart_create", "prism_dart_destroy", "prism_dart_set_round", "prism_dart_set_time",
    "prism_dart_admit", "prism_dart_commit", "prism_dart_release", "prism_dart_evict", "prism_dart_peek",
    "prism_dart_get_stats", "prism_dart_dump", "prism_dart_evicted_log", "prism_dart_check",
)

i32, i64, u64, f64 = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_double


class QasOptions(ctypes.Structure):
    _fields_ = [("dispatch_budget", i32), ("cold_quota", i32), ("front_width", i32), ("signature_size", i32),
                ("mode", i32), ("reserved", i32 * 3), ("w_global", f64), ("w_active", f64), ("w_next", f64),
                ("alpha_size", f64), ("beta_util", f64)]


class QasHint(ctypes.Structure):
    _fields_ = [("request", i64), ("bucket", u64), ("bucket_order", i32), ("rank", i32), ("lane", i32),
                ("num_segments", i32), ("first", i32), ("reserved", i32), ("bucket_score", f64), ("arrival", f64)]


class QasSegment(ctypes.Structure):
    _fields_ = [("segment", i32), ("end_offset", i32), ("g", i32), ("a", i32), ("n", i32), ("reserved", i32),
                ("priority", f64)]


class QasPriority(ctypes.Structure):
    _fields_ = [("segment", i32), ("g", i32), ("a", i32), ("n", i32), ("priority", f64)]


class DartOptions(ctypes.Structure):
    _fields_ = [("num_pages", i32), ("page_size", i32), ("policy", i32), ("protect_budget", i32),
                ("first_page", i32), ("share_in_wave", i32), ("reserved", i32 * 2)]


class DartAnchor(ctypes.Structure):
    _fields_ = [("end_offset", i32), ("kind", i32), ("segment", i32)]


class DartStats(ctypes.Structure):
    _fields_ = [("num_pages", i32), ("free_pages", i32), ("tree_pages", i32), ("private_pages", i32),
                ("num_nodes", i32), ("evictable_nodes", i32), ("locked_nodes", i32), ("protected_nodes", i32),
                ("admitted_requests", i64), ("admitted_tokens", i64), ("hit_tokens", i64),
                ("in_wave_hit_tokens", i64),
                ("evicted_pages", i64), ("evicted_nodes", i64), ("evicted_by_class", i64 * 3),
                ("heap_pops", i64), ("heap_stale", i64), ("heap_rebuilds", i64)]


class DartNode(ctypes.Structure):
    _fields_ = [("id", i32), ("parent", i32), ("num_pages", i32), ("ref", i32), ("kind", i32), ("segment", i32),
                ("num_children", i32), ("is_protected", i32), ("end_offset", i32), ("hits", ctypes.c_uint32),
                ("last", f64), ("priority", f64)]


_ready = False


def _lib():
    global _ready
    lib = B.load()
    if _ready:
        return lib
    vp, P = ctypes.c_void_p, ctypes.POINTER
    lib.prism_qas_create.argtypes = [P(QasOptions), P(vp)]
    lib.prism_qas_destroy.argtypes = [vp]
    lib.prism_qas_destroy.restype = None
    lib.prism_qas_submit.argtypes = [vp, i64, f64, P(i32), P(i32), P(ctypes.c_uint8), i32, i32, i32]
    lib.prism_qas_complete.argtypes = [vp, i64]
    lib.prism_qas_round.argtypes = [vp]
    lib.prism_qas_round_hints.argtypes = [vp, P(QasHint), i32]
    lib.prism_qas_round_segments.argtypes = [vp, P(QasSegment), i32]
    lib.prism_qas_round_priorities.argtypes = [vp, P(QasPriority), i32]
    lib.prism_qas_pending.argtypes = [vp]
    lib.prism_qas_active.argtypes = [vp]
    lib.prism_dart_create.argtypes = [P(DartOptions), P(vp)]
    lib.prism_dart_destroy.argtypes = [vp]
    lib.prism_dart_destroy.restype = None
    lib.prism_dart_set_round.argtypes = [vp, f64, P(QasPriority), i32]
    lib.prism_dart_set_time.argtypes = [vp, f64]
    lib.prism_dart_admit.argtypes = [vp, i64, P(i32), i32, P(DartAnchor), i32, i32, P(i32), i32, P(i32)]
    lib.prism_dart_commit.argtypes = [vp, i64, P(i32), i32]
    lib.prism_dart_release.argtypes = [vp, i64]
    lib.prism_dart_evict.argtypes = [vp, i32, P(i32)]
    lib.prism_dart_peek.argtypes = [vp, P(i32), i32]
    lib.prism_dart_get_stats.argtypes = [vp, P(DartStats)]
    lib.prism_dart_dump.argtypes = [vp, P(DartNode), i32]
    lib.prism_dart_evicted_log.argtypes = [vp, P(i32), i32, ctypes.c_int]
    lib.prism_dart_check.argtypes = [vp]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if fn.restype is not None:
            fn.restype = ctypes.c_int
    _ready = True
    return lib


def _check(code: int, where: str) -> int:
    if code < 0:
        raise B.PrismError(code, where)
    return code


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _p32(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(i32))


class Qas:
    """The scheduler of Sec. 3.2 / Alg. 1 (one object = one request stream)."""

    def __init__(self, dispatch_budget: int, cold_quota: int = -1, front_width: int = 0, signature_size: int = 0,
                 mode: int = QAS_MODE_QAS, weights: Optional[Tuple[float, float, float]] = None,
                 score_weights: Optional[Tuple[float, float]] = None):
        lib = _lib()
        o = QasOptions(dispatch_budget=dispatch_budget, cold_quota=cold_quota, front_width=front_width,
                       signature_size=signature_size, mode=mode)
        if weights:
            o.w_global, o.w_active, o.w_next = weights
        if score_weights:
            o.alpha_size, o.beta_util = score_weights
        self._h = ctypes.c_void_p()
        _check(lib.prism_qas_create(ctypes.byref(o), ctypes.byref(self._h)), "prism_qas_create")

    def close(self):
        if getattr(self, "_h", None) and self._h.value:
            _lib().prism_qas_destroy(self._h)
            self._h = ctypes.c_void_p()

    __del__ = close

    def submit(self, request: int, arrival: float, skeleton: Sequence[int], segment_tokens: Sequence[int],
               reorderable: Optional[Sequence[int]] = None, system_tokens: int = 0, suffix_tokens: int = 0):
        sk, st = _i32(skeleton), _i32(segment_tokens)
        ro = None
        if reorderable is not None:
            ro_a = np.ascontiguousarray(np.asarray(reorderable, dtype=np.uint8))
            ro = ro_a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))
        _check(_lib().prism_qas_submit(self._h, request, float(arrival), _p32(sk), _p32(st), ro, len(sk),
                                       system_tokens, suffix_tokens), "prism_qas_submit")

    def complete(self, request: int):
        _check(_lib().prism_qas_complete(self._h, request), "prism_qas_complete")

    def round(self):
        """Run one round; returns (hints, segments, priorities) as ctypes arrays."""
        lib = _lib()
        n = _check(lib.prism_qas_round(self._h), "prism_qas_round")
        hints = (QasHint * max(n, 1))()
        _check(lib.prism_qas_round_hints(self._h, hints, n), "prism_qas_round_hints")
        ns = _check(lib.prism_qas_round_segments(self._h, None, 0), "prism_qas_round_segments")
        segs = (QasSegment * max(ns, 1))()
        lib.prism_qas_round_segments(self._h, segs, ns)
        npri = _check(lib.prism_qas_round_priorities(self._h, None, 0), "prism_qas_round_priorities")
        pri = (QasPriority * max(npri, 1))()
        lib.prism_qas_round_priorities(self._h, pri, npri)
        return list(hints[:n]), list(segs[:ns]), (pri, npri)

    @property
    def pending(self) -> int:
        return _lib().prism_qas_pending(self._h)

    @property
    def active(self) -> int:
        return _lib().prism_qas_active(self._h)


class Dart:
    """The radix tree over cached pages with Eq. 13 / Alg. 2 eviction."""

    def __init__(self, num_pages: int, policy: int = EVICT_DART, protect_budget: int = 0, page_size: int = 16,
                 first_page: int = 0, share_in_wave: bool = False):
        lib = _lib()
        o = DartOptions(num_pages=num_pages, page_size=page_size, policy=policy, protect_budget=protect_budget,
                        first_page=first_page, share_in_wave=int(share_in_wave))
        self.page_size = page_size
        self._h = ctypes.c_void_p()
        _check(lib.prism_dart_create(ctypes.byref(o), ctypes.byref(self._h)), "prism_dart_create")

    def close(self):
        if getattr(self, "_h", None) and self._h.value:
            _lib().prism_dart_destroy(self._h)
            self._h = ctypes.c_void_p()

    __del__ = close

    def set_round(self, now: float, priorities=None):
        if priorities is None:
            arr, n = None, 0
        elif isinstance(priorities, tuple):
            arr, n = priorities
        else:  # iterable of (segment, g, a, n, priority)
            rows = list(priorities)
            n = len(rows)
            arr = (QasPriority * max(n, 1))()
            for i, (s, g, a, nn, p) in enumerate(rows):
                arr[i] = QasPriority(s, g, a, nn, p)
        _check(_lib().prism_dart_set_round(self._h, float(now), arr, n), "prism_dart_set_round")

    def set_time(self, now: float):
        _check(_lib().prism_dart_set_time(self._h, float(now)), "prism_dart_set_time")

    def admit(self, request: int, tokens, anchors: Sequence[Tuple[int, int, int]] = (), reserve_tokens: int = 0):
        """Returns (hit_tokens, block_row ndarray)."""
        tok = _i32(tokens)
        pages = (len(tok) + reserve_tokens + self.page_size - 1) // self.page_size
        row = np.full(max(pages, 1), -1, dtype=np.int32)
        an = (DartAnchor * max(len(anchors), 1))()
        for i, (off, kind, seg) in enumerate(anchors):
            an[i] = DartAnchor(off, kind, seg)
        hit = i32(0)
        _check(_lib().prism_dart_admit(self._h, request, _p32(tok), len(tok), an, len(anchors), reserve_tokens,
                                       _p32(row), len(row), ctypes.byref(hit)), "prism_dart_admit")
        return hit.value, row

    def commit(self, request: int, row: np.ndarray) -> np.ndarray:
        _check(_lib().prism_dart_commit(self._h, request, _p32(row), len(row)), "prism_dart_commit")
        return row

    def release(self, request: int):
        _check(_lib().prism_dart_release(self._h, request), "prism_dart_release")

    def evict(self, k_free_tokens: int) -> Tuple[int, int]:
        freed = i32(0)
        n = _check(_lib().prism_dart_evict(self._h, k_free_tokens, ctypes.byref(freed)), "prism_dart_evict")
        return n, freed.value

    def peek(self, tokens) -> int:
        tok = _i32(tokens)
        return _check(_lib().prism_dart_peek(self._h, _p32(tok), len(tok)), "prism_dart_peek")

    def stats(self) -> DartStats:
        s = DartStats()
        _check(_lib().prism_dart_get_stats(self._h, ctypes.byref(s)), "prism_dart_get_stats")
        return s

    def dump(self) -> List[DartNode]:
        lib = _lib()
        n = _check(lib.prism_dart_dump(self._h, None, 0), "prism_dart_dump")
        arr = (DartNode * max(n, 1))()
        lib.prism_dart_dump(self._h, arr, n)
        return list(arr[:n])

    def evicted_log(self, clear: bool = True) -> List[int]:
        lib = _lib()
        n = _check(lib.prism_dart_evicted_log(self._h, None, 0, 0), "prism_dart_evicted_log")
        arr = (i32 * max(n, 1))()
        lib.prism_dart_evicted_log(self._h, arr, n, 1 if clear else 0)
        return list(arr[:n])

    def check(self):
        _check(_lib().prism_dart_check(self._h), "prism_dart_check")
