"""ctypes wrapper around ca_oracle.c (marshalling only; all arithmetic is in the C file).

TEST INFRASTRUCTURE ONLY: see the header of ca_oracle.c.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ca_oracle.c")
_LIB = os.path.join(_HERE, "libca_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64, OpenMP over query heads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-ffp-contract=off", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            build()
            lib = C.CDLL(_LIB)
            dp, ip, bp = C.POINTER(C.c_double), C.POINTER(C.c_int32), C.c_void_p
            lib.cao_rope.argtypes = [dp, C.c_int, C.c_double, C.c_double, C.c_int, dp]
            lib.cao_rope.restype = None
            lib.cao_attention_positions.argtypes = [dp, dp, C.c_int, dp, C.c_int, dp, dp, C.c_int,
                                                    C.c_int, C.c_int, C.c_int, C.c_double, C.c_int,
                                                    C.c_double, dp, dp]
            lib.cao_attention_positions.restype = C.c_int
            lib.cao_cached_attention.argtypes = [dp, dp, C.c_int, dp, dp, dp, C.c_int, C.c_int,
                                                 C.c_int, C.c_int, C.c_int, C.c_double, C.c_int,
                                                 C.c_double, C.c_double, dp, dp]
            lib.cao_cached_attention.restype = C.c_int
            lib.cao_truncate_plan.argtypes = [ip, ip, C.c_int32, C.c_double, C.c_int, C.c_int, ip]
            lib.cao_truncate_plan.restype = C.c_int
            lib.cao_rebase.argtypes = [C.c_int, ip, ip, ip, ip, C.c_int, C.c_int,
                                       ip, ip, ip, ip, ip, ip]
            lib.cao_rebase.restype = C.c_int
            lib.cao_unpack.argtypes = [bp, C.c_int64, bp, ip, C.c_int, C.c_int, C.c_int, C.c_int,
                                       C.c_int, C.c_int]
            lib.cao_unpack.restype = None
            lib.cao_pack.argtypes = [bp, ip, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                     bp, C.c_int64]
            lib.cao_pack.restype = None
            lib.cao_kv_bytes_per_token.argtypes = [C.c_int] * 4
            lib.cao_kv_bytes_per_token.restype = C.c_int64
            _lib = lib
    return _lib


def n_threads() -> int:
    """Threads the OpenMP loops of the oracle will use."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


def _i(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


def _check(rc):
    if rc != 0:
        raise ValueError(f"oracle rejected its arguments (code {rc})")


def rope(x, pos: float, base: float = 10000.0, style: int = 0) -> np.ndarray:
    x, xp = _d(x)
    assert x.ndim == 1 and x.shape[0] % 2 == 0
    out = np.empty_like(x)
    _load().cao_rope(xp, x.shape[0], float(pos), float(base), int(style),
                     out.ctypes.data_as(C.POINTER(C.c_double)))
    return out


def attention_positions(K, V, Q, kpos, qpos, n: int, base=10000.0, style=0, scale=None,
                        return_probs=False):
    K, Kp = _d(K); V, Vp = _d(V); Q, Qp = _d(Q)
    Lk, Hkv, D = K.shape
    Ln, Hq, _ = Q.shape
    assert V.shape == K.shape and Q.shape[2] == D
    kpos, kpp = _d(kpos); qpos, qpp = _d(qpos)
    assert kpos.shape == (Lk,) and qpos.shape == (Ln,)
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    O = np.empty((Ln, Hq, D), dtype=np.float64)
    P = np.empty((Hq, Ln, Lk), dtype=np.float64) if return_probs else None
    rc = _load().cao_attention_positions(
        Kp, Vp, Lk, Qp, Ln, kpp, qpp, int(n), Hq, Hkv, D, float(base), int(style), float(scale),
        O.ctypes.data_as(C.POINTER(C.c_double)),
        P.ctypes.data_as(C.POINTER(C.c_double)) if P is not None else None)
    _check(rc)
    return (O, P) if return_probs else O


def cached_attention(Kh, Vh, Qn, Kn, Vn, keep_start: int = 0, base=10000.0, style=0, scale=None,
                     pos_shift: float = 0.0, return_probs=False):
    """New-turn prefill over a reused cache, one conversation, one layer (fp64)."""
    Kh, Khp = _d(Kh); Vh, Vhp = _d(Vh); Qn, Qp = _d(Qn); Kn, Knp = _d(Kn); Vn, Vnp = _d(Vn)
    Ln, Hq, D = Qn.shape
    Hkv = Kn.shape[1]
    Lh = Kh.shape[0]
    assert Kh.shape == (Lh, Hkv, D) and Vh.shape == (Lh, Hkv, D)
    assert Kn.shape == (Ln, Hkv, D) and Vn.shape == (Ln, Hkv, D)
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    Lk = Lh - int(keep_start) + Ln
    O = np.empty((Ln, Hq, D), dtype=np.float64)
    P = np.empty((Hq, Ln, max(Lk, 0)), dtype=np.float64) if return_probs else None
    rc = _load().cao_cached_attention(
        Khp, Vhp, Lh, Qp, Knp, Vnp, Ln, int(keep_start), Hq, Hkv, D, float(base), int(style),
        float(scale), float(pos_shift), O.ctypes.data_as(C.POINTER(C.c_double)),
        P.ctypes.data_as(C.POINTER(C.c_double)) if P is not None else None)
    _check(rc)
    return (O, P) if return_probs else O


def cached_attention_kept(Kh, Vh, kept, Qn, Kn, Vn, **kw):
    """Section 3.4, last paragraph: the history survives a token discarding list as the saved tokens with
    indices `kept` (increasing).  The store delivers exactly those, they are renumbered densely from 0 and
    the new turn attends to them: by definition the reuse path over the pruned history."""
    kept = np.asarray(kept, dtype=np.int64)
    assert kept.ndim == 1 and (len(kept) < 2 or np.all(np.diff(kept) > 0))
    assert len(kept) == 0 or (kept[0] >= 0 and kept[-1] < np.asarray(Kh).shape[0])
    return cached_attention(np.asarray(Kh)[kept], np.asarray(Vh)[kept], Qn, Kn, Vn, keep_start=0, **kw)


def compact_tier(rows, ranges) -> np.ndarray:
    """Section 3.4, last paragraph: the saved cache of a conversation after the discarded tokens have been
    dropped from the store: the rows of the kept ranges [(begin, end), ...] (increasing, disjoint), in order."""
    rows = np.asarray(rows)
    out = [rows[int(b):int(e)] for b, e in ranges]
    return np.concatenate(out) if out else rows[:0].copy()


def kept_indices_sinks(hist_len, new_len, window: int, ratio: float = 0.5, n_sink: int = 4) -> list:
    """Discarding list that spares the first n_sink saved tokens: without overflow everything is kept; on
    overflow (hist + new > window) the history may keep floor(window*(1-ratio)) - new tokens (not below 0,
    not above hist): the first min(n_sink, budget) and the most recent rest.  Returns, per conversation,
    the kept indices in increasing order."""
    out = []
    for h, n in zip(np.asarray(hist_len, dtype=np.int64), np.asarray(new_len, dtype=np.int64)):
        if h + n <= window:
            out.append(np.arange(h))
            continue
        budget = int(min(h, max(0, int(np.floor(window * (1.0 - ratio))) - n)))
        sinks = min(int(n_sink), budget)
        idx = set(range(sinks)) | set(range(int(h) - (budget - sinks), int(h)))
        out.append(np.array(sorted(idx), dtype=np.int64))
    return out


def truncate_plan(hist_len, new_len, window: int, ratio: float = 0.5, policy: int = 0) -> np.ndarray:
    h, hp = _i(hist_len); n, np_ = _i(new_len)
    out = np.empty(h.shape[0], dtype=np.int32)
    rc = _load().cao_truncate_plan(hp, np_, int(window), float(ratio), int(policy), h.shape[0],
                                   out.ctypes.data_as(C.POINTER(C.c_int32)))
    _check(rc)
    return out


def rebase(hist_len, keep_start, new_len, block_table, page_size: int) -> dict:
    h, hp = _i(hist_len); s, sp = _i(keep_start); n, np_ = _i(new_len)
    bt, btp = _i(block_table)
    B = h.shape[0]
    assert bt.ndim == 2 and bt.shape[0] == B
    n_keep = np.empty(B, np.int32); cu_q = np.empty(B + 1, np.int32); cu_k = np.empty(B + 1, np.int32)
    tot_q = int(np.sum(n.astype(np.int64)))
    tot_k = int(np.sum(h.astype(np.int64) - s + n))
    q_pos = np.empty(max(tot_q, 1), np.int32); q_seq = np.empty(max(tot_q, 1), np.int32)
    slot_map = np.empty(max(tot_k, 1), np.int32)
    ip = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))  # noqa: E731
    rc = _load().cao_rebase(B, hp, sp, np_, btp, bt.shape[1], int(page_size),
                            ip(n_keep), ip(cu_q), ip(cu_k), ip(q_pos), ip(q_seq), ip(slot_map))
    _check(rc)
    return dict(n_keep=n_keep, cu_q=cu_q, cu_k=cu_k, q_pos=q_pos[:tot_q], q_seq=q_seq[:tot_q],
                slot_map=slot_map[:tot_k])


def _bytes(a):
    a = np.ascontiguousarray(a)
    return a, a.ctypes.data_as(C.c_void_p)


def unpack(contig, src_tok0: int, pool, table, page_size: int, n_kv_heads: int, head_dim: int,
           dst_tok0: int, count: int) -> None:
    """contig [tokens][Hkv][D] -> pool [pages][Hkv][P][D], in place on `pool` (any dtype)."""
    assert pool.flags["C_CONTIGUOUS"] and pool.dtype == contig.dtype
    contig, cp = _bytes(contig)
    table, tp = _i(table)
    _load().cao_unpack(cp, int(src_tok0), pool.ctypes.data_as(C.c_void_p), tp, int(page_size),
                       int(n_kv_heads), int(head_dim), pool.dtype.itemsize, int(dst_tok0), int(count))


def pack(pool, table, page_size: int, n_kv_heads: int, head_dim: int, src_tok0: int, count: int,
         contig, dst_tok0: int) -> None:
    """pool -> contig, in place on `contig`."""
    assert contig.flags["C_CONTIGUOUS"] and pool.dtype == contig.dtype
    pool, pp = _bytes(pool)
    table, tp = _i(table)
    _load().cao_pack(pp, tp, int(page_size), int(n_kv_heads), int(head_dim), pool.dtype.itemsize,
                     int(src_tok0), int(count), contig.ctypes.data_as(C.c_void_p), int(dst_tok0))


def kv_bytes_per_token(n_layers: int, n_kv_heads: int, head_dim: int, esize: int = 2) -> int:
    return int(_load().cao_kv_bytes_per_token(n_layers, n_kv_heads, head_dim, esize))
