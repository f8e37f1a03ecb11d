"""ctypes binding of include/ca.h.  Argument marshalling only.

Tensors are passed as anything with .data_ptr() (torch tensors) or as integer addresses; streams
as anything with .cuda_stream (torch.cuda.Stream), an integer hipStream_t, or None for the
default stream.  Errors surface as CaError carrying the ca_status and the library's message.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, fields

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libca_hip.so")
_lib = None

STATUS = {0: "CA_OK", 1: "CA_ERR_INVALID_ARG", 2: "CA_ERR_OUT_OF_RANGE", 3: "CA_ERR_UNSUPPORTED",
          4: "CA_ERR_NOMEM", 5: "CA_ERR_NOT_READY", 6: "CA_ERR_HIP"}

# every symbol include/ca.h declares
SYMBOLS = ["ca_config_default", "ca_config_validate", "ca_batch_validate", "ca_create", "ca_destroy",
           "ca_last_error", "ca_status_string", "ca_truncate_plan", "ca_truncate_plan_sinks", "ca_rope_rebase", "ca_rebase_read",
           "ca_kv_load_layer", "ca_kv_append_layer", "ca_cached_prefill_attn", "ca_cached_prefill_attn_static",
           "ca_kv_save_layer", "ca_kv_append_save_layer",
           "ca_sync", "ca_join", "ca_profile_enable", "ca_profile_read", "ca_profile_timeline", "ca_tier_compact"]


class CaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status
        self.status_name = STATUS.get(status, str(status))


class _CConfig(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("page_size", C.c_int32), ("max_positions", C.c_int32),
                ("rope_base", C.c_float), ("rope_style", C.c_int32), ("pipeline_depth", C.c_int32),
                ("max_seqs", C.c_int32), ("max_batch_kv_tokens", C.c_int64),
                ("max_batch_q_tokens", C.c_int64), ("load_mode", C.c_int32), ("save_mode", C.c_int32),
                ("attn_variant", C.c_int32), ("attn_tile_rows", C.c_int32), ("attn_split", C.c_int32),
                ("attn_prerotate", C.c_int32), ("attn_schedule", C.c_int32), ("require_load", C.c_int32),
                ("device", C.c_int32)]


class _CBatch(C.Structure):
    _fields_ = [("n_seqs", C.c_int32), ("hist_len", C.POINTER(C.c_int32)),
                ("keep_start", C.POINTER(C.c_int32)), ("new_len", C.POINTER(C.c_int32)),
                ("block_table", C.POINTER(C.c_int32)), ("max_pages", C.c_int32),
                ("num_pages", C.c_int32), ("keep_ranges", C.POINTER(C.c_int32)),
                ("keep_range_count", C.POINTER(C.c_int32))]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libca_hip.so; raises if it has not been built.  There is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2403_19708_amd.build` "
                           "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32p, i64p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    lib.ca_config_default.argtypes = [C.POINTER(_CConfig)]
    lib.ca_config_default.restype = None
    lib.ca_config_validate.argtypes = [C.POINTER(_CConfig), C.c_char_p, C.c_int32]
    lib.ca_config_validate.restype = C.c_int
    lib.ca_batch_validate.argtypes = [C.POINTER(_CConfig), C.POINTER(_CBatch), C.c_char_p, C.c_int32]
    lib.ca_batch_validate.restype = C.c_int
    lib.ca_create.argtypes = [C.POINTER(_CConfig), C.POINTER(vp)]
    lib.ca_create.restype = C.c_int
    lib.ca_destroy.argtypes = [vp]
    lib.ca_destroy.restype = None
    lib.ca_last_error.argtypes = [vp]
    lib.ca_last_error.restype = C.c_char_p
    lib.ca_status_string.argtypes = [C.c_int]
    lib.ca_status_string.restype = C.c_char_p
    lib.ca_truncate_plan.argtypes = [i32p, i32p, C.c_int32, C.c_double, C.c_int32, C.c_int32, i32p]
    lib.ca_truncate_plan.restype = C.c_int
    lib.ca_truncate_plan_sinks.argtypes = [i32p, i32p, C.c_int32, C.c_double, C.c_int32, C.c_int32, i32p, i32p]
    lib.ca_truncate_plan_sinks.restype = C.c_int
    lib.ca_rope_rebase.argtypes = [vp, C.POINTER(_CBatch), vp]
    lib.ca_rope_rebase.restype = C.c_int
    lib.ca_rebase_read.argtypes = [vp, C.c_int32, i32p, C.c_int64, i64p]
    lib.ca_rebase_read.restype = C.c_int
    lib.ca_kv_load_layer.argtypes = [vp, C.c_int32, C.POINTER(vp), C.POINTER(vp), vp, vp]
    lib.ca_kv_load_layer.restype = C.c_int
    lib.ca_kv_append_layer.argtypes = [vp, C.c_int32, vp, vp, vp, vp, vp]
    lib.ca_kv_append_layer.restype = C.c_int
    lib.ca_cached_prefill_attn.argtypes = [vp, C.c_int32, vp, vp, vp, vp, C.c_float, vp]
    lib.ca_cached_prefill_attn.restype = C.c_int
    lib.ca_cached_prefill_attn_static.argtypes = [vp, C.c_int32, vp, vp, vp, vp, C.c_float, vp]
    lib.ca_cached_prefill_attn_static.restype = C.c_int
    # the three optional per-conversation arrays go in as plain addresses (cheaper to marshal per call)
    lib.ca_kv_save_layer.argtypes = [vp, C.c_int32, vp, vp, vp, vp, C.POINTER(vp), C.POINTER(vp), vp, vp]
    lib.ca_kv_save_layer.restype = C.c_int
    lib.ca_kv_append_save_layer.argtypes = [vp, C.c_int32, vp, vp, vp, vp, C.POINTER(vp), C.POINTER(vp), vp]
    lib.ca_kv_append_save_layer.restype = C.c_int
    lib.ca_sync.argtypes = [vp]
    lib.ca_sync.restype = C.c_int
    lib.ca_join.argtypes = [vp, vp]
    lib.ca_join.restype = C.c_int
    lib.ca_profile_enable.argtypes = [vp, C.c_int32]
    lib.ca_profile_enable.restype = C.c_int
    lib.ca_profile_read.argtypes = [vp, C.c_int32, C.POINTER(C.c_double), i64p]
    lib.ca_profile_read.restype = C.c_int
    lib.ca_profile_timeline.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_int64, i64p]
    lib.ca_profile_timeline.restype = C.c_int
    lib.ca_tier_compact.argtypes = [C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                    C.c_int64, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_int32)]
    lib.ca_tier_compact.restype = C.c_int
    _lib = lib
    return lib


@dataclass
class Config:
    n_layers: int = 1
    n_q_heads: int = 1
    n_kv_heads: int = 1
    head_dim: int = 128
    page_size: int = 16
    max_positions: int = 4096
    rope_base: float = 10000.0
    rope_style: int = 0
    pipeline_depth: int = 2
    max_seqs: int = 64
    max_batch_kv_tokens: int = 1 << 16
    max_batch_q_tokens: int = 1 << 14
    load_mode: int = 0
    save_mode: int = 0
    attn_variant: int = 0
    attn_tile_rows: int = 0
    attn_split: int = 0
    attn_prerotate: int = 0
    attn_schedule: int = 0
    require_load: int = 1
    device: int = 0

    def to_c(self) -> _CConfig:
        c = _CConfig()
        for f in fields(self):
            setattr(c, f.name, getattr(self, f.name))
        return c


def _ptr(x) -> int:
    if x is None:
        return 0
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    return int(x)


def _stream(s) -> int:
    if s is None:
        return 0
    if hasattr(s, "cuda_stream"):
        return int(s.cuda_stream)
    return int(s)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


def pointer_array(ptrs):
    """One pointer per conversation as the C array the load/save calls take.  The calls accept the result in
    place of the list, so a caller that passes the same pointers again and again builds it once."""
    if isinstance(ptrs, C.Array):
        return ptrs
    return (C.c_void_p * len(ptrs))(*[_ptr(p) or None for p in ptrs])


def _make_batch(hist_len, keep_start, new_len, block_table, num_pages, keep_ranges=None):
    """keep_ranges: None, or one list of (begin, end) pairs per conversation (then keep_start may be None)."""
    h, hp = _i32(hist_len)
    s, sp = _i32(keep_start) if keep_start is not None else (None, None)
    n, np_ = _i32(new_len)
    bt, btp = _i32(block_table)
    if bt.ndim != 2:
        raise ValueError("block_table must be [n_seqs][max_pages]")
    rng = cnt = rp = cp = None
    if keep_ranges is not None:
        if len(keep_ranges) != h.shape[0]:
            raise ValueError("keep_ranges needs one list of (begin, end) pairs per conversation")
        cnt, cp = _i32([len(r) for r in keep_ranges])
        flat = [pair for r in keep_ranges for pair in r]
        rng, rp = _i32(np.asarray(flat, dtype=np.int32).reshape(-1, 2) if flat else np.zeros((1, 2), np.int32))
    b = _CBatch(h.shape[0], hp, sp, np_, btp, bt.shape[1], int(num_pages), rp, cp)
    return b, (h, s, n, bt, rng, cnt)


def config_validate(cfg: Config) -> None:
    lib = load_library()
    buf = C.create_string_buffer(512)
    c = cfg.to_c()
    st = lib.ca_config_validate(C.byref(c), buf, 512)
    if st != 0:
        raise CaError(st, buf.value.decode())


def batch_validate(cfg: Config, hist_len, keep_start, new_len, block_table, num_pages, keep_ranges=None) -> None:
    lib = load_library()
    buf = C.create_string_buffer(512)
    c = cfg.to_c()
    b, keep = _make_batch(hist_len, keep_start, new_len, block_table, num_pages, keep_ranges)
    st = lib.ca_batch_validate(C.byref(c), C.byref(b), buf, 512)
    del keep
    if st != 0:
        raise CaError(st, buf.value.decode())


def truncate_plan(hist_len, new_len, window: int, ratio: float = 0.5, policy: int = 0) -> np.ndarray:
    lib = load_library()
    h, hp = _i32(hist_len)
    n, np_ = _i32(new_len)
    if h.shape != n.shape or h.ndim != 1:
        raise ValueError("hist_len and new_len must be 1-D and equally long")
    out = np.zeros(h.shape[0], dtype=np.int32)
    st = lib.ca_truncate_plan(hp, np_, int(window), float(ratio), int(policy), h.shape[0],
                              out.ctypes.data_as(C.POINTER(C.c_int32)))
    if st != 0:
        raise CaError(st, "ca_truncate_plan rejected its arguments")
    return out


def truncate_plan_sinks(hist_len, new_len, window: int, ratio: float = 0.5, n_sink: int = 4) -> list:
    """One list of (begin, end) kept ranges per conversation (the shape ca_batch.keep_ranges takes)."""
    lib = load_library()
    h, hp = _i32(hist_len)
    n, np_ = _i32(new_len)
    if h.shape != n.shape or h.ndim != 1:
        raise ValueError("hist_len and new_len must be 1-D and equally long")
    rng = np.zeros((h.shape[0], 2, 2), dtype=np.int32)
    cnt = np.zeros(h.shape[0], dtype=np.int32)
    st = lib.ca_truncate_plan_sinks(hp, np_, int(window), float(ratio), int(n_sink), h.shape[0],
                                    rng.ctypes.data_as(C.POINTER(C.c_int32)), cnt.ctypes.data_as(C.POINTER(C.c_int32)))
    if st != 0:
        raise CaError(st, "ca_truncate_plan_sinks rejected its arguments")
    return [[(int(rng[c, r, 0]), int(rng[c, r, 1])) for r in range(int(cnt[c]))] for c in range(h.shape[0])]


def tier_compact(hist_len, keep, row_bytes: int, tier_k, tier_v) -> np.ndarray:
    """Drops the discarded rows of one layer's saved cache in host memory (ca_tier_compact).  keep: per conversation
    either a keep_start (int) or a list of (begin, end) kept ranges; tier_k / tier_v: per conversation a host address
    (int) or an object with data_ptr() (a CPU or pinned torch tensor).  Returns the new history lengths."""
    lib = load_library()
    h, hp = _i32(hist_len)
    n = h.shape[0]
    if len(keep) != n or len(tier_k) != n or len(tier_v) != n:
        raise ValueError("one entry per conversation expected")
    ptr = lambda t: int(t.data_ptr()) if hasattr(t, "data_ptr") else int(t)
    pk = (C.c_void_p * n)(*[ptr(t) for t in tier_k])
    pv = (C.c_void_p * n)(*[ptr(t) for t in tier_v])
    out = np.zeros(n, dtype=np.int32)
    i32p = C.POINTER(C.c_int32)
    if all(isinstance(k, (int, np.integer)) for k in keep):
        ks, ksp = _i32(keep)
        st = lib.ca_tier_compact(n, hp, ksp, None, None, int(row_bytes), pk, pv, out.ctypes.data_as(i32p))
    else:
        flat = np.array([x for rs in keep for r in rs for x in r], dtype=np.int32).reshape(-1)
        cnt = np.array([len(rs) for rs in keep], dtype=np.int32)
        st = lib.ca_tier_compact(n, hp, None, flat.ctypes.data_as(i32p) if flat.size else (C.c_int32 * 1)(), cnt.ctypes.data_as(i32p),
                                 int(row_bytes), pk, pv, out.ctypes.data_as(i32p))
    if st != 0:
        raise CaError(st, "ca_tier_compact rejected its arguments")
    return out


class Context:
    """Owns one ca_ctx.  Method names follow the C entry points without the ca_ prefix."""

    def __init__(self, cfg: Config):
        self._lib = load_library()
        self.cfg = cfg
        self._h = C.c_void_p()
        c = cfg.to_c()
        st = self._lib.ca_create(C.byref(c), C.byref(self._h))
        if st != 0:
            self._h = C.c_void_p()
            buf = C.create_string_buffer(512)
            self._lib.ca_config_validate(C.byref(c), buf, 512)
            raise CaError(st, buf.value.decode() or "ca_create failed (see stderr)")
        self.n_seqs = 0

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.ca_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def _check(self, st: int):
        if st != 0:
            raise CaError(st, self._lib.ca_last_error(self._h).decode())

    # ---- Section 3.4 ------------------------------------------------------------------------
    def rope_rebase(self, hist_len, keep_start, new_len, block_table, num_pages: int, stream=None, keep_ranges=None):
        b, keep = _make_batch(hist_len, keep_start, new_len, block_table, num_pages, keep_ranges)
        st = self._lib.ca_rope_rebase(self._h, C.byref(b), _stream(stream))
        del keep
        self._check(st)
        self.n_seqs = b.n_seqs

    def rebase_read(self, which: int, capacity: int | None = None) -> np.ndarray:
        cap = int(capacity) if capacity is not None else int(
            max(self.cfg.max_batch_kv_tokens, 8 * (self.cfg.max_batch_q_tokens + 16384)))
        out = np.empty(cap, dtype=np.int32)
        cnt = C.c_int64(0)
        self._check(self._lib.ca_rebase_read(self._h, int(which), out.ctypes.data_as(C.POINTER(C.c_int32)),
                                             cap, C.byref(cnt)))
        return out[:cnt.value].copy()

    # ---- Section 3.2.1 ----------------------------------------------------------------------
    def _ptr_array(self, ptrs):
        return pointer_array(ptrs)

    def kv_load_layer(self, layer: int, src_k, src_v, k_pool, v_pool):
        ak, av = self._ptr_array(src_k), self._ptr_array(src_v)
        if self.n_seqs and (len(ak) != self.n_seqs or len(av) != self.n_seqs):
            raise ValueError("src_k/src_v need one pointer per conversation of the current plan")
        self._check(self._lib.ca_kv_load_layer(self._h, int(layer), ak, av, _ptr(k_pool), _ptr(v_pool)))

    def kv_append_layer(self, layer: int, new_k, new_v, k_pool, v_pool, stream=None):
        self._check(self._lib.ca_kv_append_layer(self._h, int(layer), _ptr(new_k), _ptr(new_v),
                                                 _ptr(k_pool), _ptr(v_pool), _stream(stream)))

    # ---- Sections 2.1 / 3.1 / 3.4 -----------------------------------------------------------
    def cached_prefill_attn(self, layer: int, q, k_pool, v_pool, out, softmax_scale: float, stream=None):
        self._check(self._lib.ca_cached_prefill_attn(self._h, int(layer), _ptr(q), _ptr(k_pool), _ptr(v_pool),
                                                     _ptr(out), float(softmax_scale), _stream(stream)))

    def cached_prefill_attn_static(self, layer: int, q, k_pool, v_pool, out, softmax_scale: float, stream=None):
        self._check(self._lib.ca_cached_prefill_attn_static(self._h, int(layer), _ptr(q), _ptr(k_pool), _ptr(v_pool),
                                                            _ptr(out), float(softmax_scale), _stream(stream)))

    # ---- Section 3.2.2 ----------------------------------------------------------------------
    def kv_save_layer(self, layer: int, k_pool, v_pool, dst_k, dst_v, tok_begin=None, tok_end=None,
                      dst_tok_offset=None, after_stream=None):
        ak, av = self._ptr_array(dst_k), self._ptr_array(dst_v)
        if self.n_seqs and (len(ak) != self.n_seqs or len(av) != self.n_seqs):
            raise ValueError("dst_k/dst_v need one pointer per conversation of the current plan")
        keep = []
        def opt(a, dtype):
            if a is None:
                return None
            arr = np.ascontiguousarray(a, dtype=dtype)
            if arr.shape != (self.n_seqs,):
                raise ValueError("per-conversation arrays must have n_seqs entries")
            keep.append(arr)
            return arr.ctypes.data
        tb, te, off = opt(tok_begin, np.int32), opt(tok_end, np.int32), opt(dst_tok_offset, np.int64)
        self._check(self._lib.ca_kv_save_layer(self._h, int(layer), tb, te, _ptr(k_pool), _ptr(v_pool), ak, av,
                                               off, _stream(after_stream)))

    def kv_append_save_layer(self, layer: int, new_k, new_v, k_pool, v_pool, dst_k, dst_v, stream=None):
        ak, av = self._ptr_array(dst_k), self._ptr_array(dst_v)
        if self.n_seqs and (len(ak) != self.n_seqs or len(av) != self.n_seqs):
            raise ValueError("dst_k/dst_v need one pointer per conversation of the current plan")
        self._check(self._lib.ca_kv_append_save_layer(self._h, int(layer), _ptr(new_k), _ptr(new_v), _ptr(k_pool),
                                                      _ptr(v_pool), ak, av, _stream(stream)))

    def sync(self):
        self._check(self._lib.ca_sync(self._h))

    def join(self, stream=None):
        self._check(self._lib.ca_join(self._h, _stream(stream)))

    PROFILE_KINDS = {"copy_in": 0, "unpack": 1, "append": 2, "attn": 3, "pack": 4, "copy_out": 5}

    def profile_enable(self, on: bool = True, kinds=None):
        """kinds: None = every kind, else an iterable of kind names/numbers to time"""
        arg = 1 if on else 0
        if on and kinds is not None:
            mask = 0
            for k in kinds:
                mask |= 1 << (self.PROFILE_KINDS[k] if isinstance(k, str) else int(k))
            arg = 2 * mask
        self._check(self._lib.ca_profile_enable(self._h, arg))

    def profile_read(self, kind) -> tuple[float, int]:
        """(summed milliseconds, number of intervals) of one kind since the last read."""
        k = self.PROFILE_KINDS[kind] if isinstance(kind, str) else int(kind)
        ms, n = C.c_double(0.0), C.c_int64(0)
        self._check(self._lib.ca_profile_read(self._h, k, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def profile_timeline(self):
        """[(kind name, start ms, stop ms)] of the intervals not read yet, on one clock (zero = the first one's start)."""
        n = C.c_int64(0)
        self._check(self._lib.ca_profile_timeline(self._h, None, None, None, 0, C.byref(n)))
        cap = n.value
        if cap == 0:
            return []
        kinds, t0, t1 = (C.c_int32 * cap)(), (C.c_double * cap)(), (C.c_double * cap)()
        self._check(self._lib.ca_profile_timeline(self._h, kinds, t0, t1, cap, C.byref(n)))
        names = {v: k for k, v in self.PROFILE_KINDS.items()}
        return [(names[kinds[i]], t0[i], t1[i]) for i in range(min(cap, n.value))]
