"""ctypes binding of include/ca_store.h (the placement manager of Section 3.3).  Argument marshalling
only: every decision is taken in the library."""
from __future__ import annotations

import ctypes as C

import numpy as np

from .binding import CaError, load_library

SCHEDULER_AWARE, LRU, FIFO = 0, 1, 2
MISS, HIT_MEM, HIT_DISK = 0, 1, 2
IN_MEM, ON_DISK = 1, 2
FETCH, LOAD, EVICT, RELEASE, DROP_DISK, DROP, EXPIRE = 1, 2, 3, 4, 5, 6, 7

# every symbol include/ca_store.h declares
SYMBOLS = ["ca_store_create", "ca_store_destroy", "ca_store_last_error", "ca_store_seed", "ca_store_set_queue",
           "ca_store_prefetch", "ca_store_lookup", "ca_store_save", "ca_store_release", "ca_store_where", "ca_store_windows",
           "ca_store_usage", "ca_store_stats_read", "ca_store_take_actions"]


class _CStoreConfig(C.Structure):
    _fields_ = [("mem_capacity", C.c_int64), ("disk_capacity", C.c_int64), ("mem_buffer", C.c_int64),
                ("policy", C.c_int32), ("prefetch", C.c_int32), ("ttl", C.c_double)]


class _CAction(C.Structure):
    _fields_ = [("kind", C.c_int32), ("reserved", C.c_int32), ("session", C.c_int64)]


STAT_FIELDS = ["lookups", "hit_mem", "hit_disk", "miss", "fetched", "loaded", "evicted", "released", "dropped",
               "expired", "forced_window_drops", "bytes_to_disk", "bytes_from_disk"]


class _CStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in STAT_FIELDS]


_ready = False


def _lib():
    global _ready
    lib = load_library()
    if not _ready:
        vp, i64p, i32p = C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int32)
        lib.ca_store_create.argtypes = [C.POINTER(_CStoreConfig), C.POINTER(vp)]
        lib.ca_store_destroy.argtypes = [vp]
        lib.ca_store_destroy.restype = None
        lib.ca_store_last_error.argtypes = [vp]
        lib.ca_store_last_error.restype = C.c_char_p
        lib.ca_store_seed.argtypes = [vp, C.c_int64, C.c_int64, C.c_int32, C.c_double]
        lib.ca_store_set_queue.argtypes = [vp, i64p, C.c_int32]
        lib.ca_store_prefetch.argtypes = [vp, C.c_double]
        lib.ca_store_lookup.argtypes = [vp, C.c_int64, C.c_double, i32p]
        lib.ca_store_save.argtypes = [vp, C.c_int64, C.c_int64, C.c_double]
        lib.ca_store_release.argtypes = [vp, C.c_int64, C.c_double]
        lib.ca_store_where.argtypes = [vp, C.c_int64, i32p]
        lib.ca_store_windows.argtypes = [vp, i64p, i64p]
        lib.ca_store_usage.argtypes = [vp, i64p, i64p, i64p]
        lib.ca_store_stats_read.argtypes = [vp, C.POINTER(_CStats)]
        lib.ca_store_take_actions.argtypes = [vp, C.POINTER(_CAction), C.c_int64, i64p]
        for n in SYMBOLS:
            if n not in ("ca_store_destroy", "ca_store_last_error"):
                getattr(lib, n).restype = C.c_int
        _ready = True
    return lib


class Store:
    """One placement manager.  Use as a context manager or call close()."""

    def __init__(self, mem_capacity, disk_capacity, mem_buffer=0, policy=SCHEDULER_AWARE, prefetch=True, ttl=0.0):
        self._lib = _lib()
        cfg = _CStoreConfig(int(mem_capacity), int(disk_capacity), int(mem_buffer), int(policy), int(bool(prefetch)), float(ttl))
        h = C.c_void_p()
        st = self._lib.ca_store_create(C.byref(cfg), C.byref(h))
        if st != 0:
            raise CaError(st, "ca_store_create rejected the configuration")
        self._h = h

    def _check(self, st):
        if st != 0:
            raise CaError(st, self._lib.ca_store_last_error(self._h).decode())

    def close(self):
        if self._h:
            self._lib.ca_store_destroy(self._h)
            self._h = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def seed(self, session, size, tiers, now=0.0):
        self._check(self._lib.ca_store_seed(self._h, int(session), int(size), int(tiers), float(now)))

    def set_queue(self, sessions):
        a = np.ascontiguousarray(sessions, dtype=np.int64)
        self._check(self._lib.ca_store_set_queue(self._h, a.ctypes.data_as(C.POINTER(C.c_int64)), len(a)))

    def prefetch(self, now):
        self._check(self._lib.ca_store_prefetch(self._h, float(now)))

    def lookup(self, session, now) -> int:
        out = C.c_int32()
        self._check(self._lib.ca_store_lookup(self._h, int(session), float(now), C.byref(out)))
        return out.value

    def save(self, session, size, now):
        self._check(self._lib.ca_store_save(self._h, int(session), int(size), float(now)))

    def release(self, session, now):
        self._check(self._lib.ca_store_release(self._h, int(session), float(now)))

    def where(self, session) -> int:
        out = C.c_int32()
        self._check(self._lib.ca_store_where(self._h, int(session), C.byref(out)))
        return out.value

    def windows(self) -> tuple[int, int]:
        a, b = C.c_int64(), C.c_int64()
        self._check(self._lib.ca_store_windows(self._h, C.byref(a), C.byref(b)))
        return a.value, b.value

    def usage(self) -> tuple[int, int, int]:
        a, b, n = C.c_int64(), C.c_int64(), C.c_int64()
        self._check(self._lib.ca_store_usage(self._h, C.byref(a), C.byref(b), C.byref(n)))
        return a.value, b.value, n.value

    def stats(self) -> dict:
        s = _CStats()
        self._check(self._lib.ca_store_stats_read(self._h, C.byref(s)))
        return {n: getattr(s, n) for n in STAT_FIELDS}

    def take_actions(self) -> list[tuple[int, int]]:
        n = C.c_int64()
        st = self._lib.ca_store_take_actions(self._h, None, 0, C.byref(n))
        if st == 0:
            return []
        buf = (_CAction * n.value)()
        self._check(self._lib.ca_store_take_actions(self._h, buf, n.value, C.byref(n)))
        return [(a.kind, a.session) for a in buf[:n.value]]
