"""Pins for the fp64 oracle's attention, written against what the paper and the mathematics fix,
not against the oracle's own formulas.  CPU only.

The independent reference below uses a different formulation on purpose: rotary pairs as complex
numbers multiplied by exp(i p theta), one dense causal attention over the WHOLE context with
einsum, scipy's logsumexp.  It recomputes what a serving engine without the cache would compute
(Section 2.3: the history is prefilled again), so "reuse == recompute" (Section 3.1) is the test.
"""
import numpy as np
import pytest
import torch
from scipy.special import logsumexp

import oracle
from synth import bf16_bits_to_f64, draw_values_bf16


def rot_complex(x, pos, base=10000.0):
    """x [..., L, H, D] rotated at pos [L]; half-split pairs as complex numbers."""
    D = x.shape[-1]
    half = D // 2
    z = x[..., :half] + 1j * x[..., half:]
    theta = base ** (-np.arange(half) * 2.0 / D)
    ph = np.exp(1j * np.asarray(pos, dtype=np.float64)[:, None, None] * theta)
    z = z * ph
    return np.concatenate([z.real, z.imag], axis=-1)


def full_recompute(Q, K, V, base=10000.0, first_pos=0):
    """Plain causal attention over all L tokens: Q [L][Hq][D], K,V [L][Hkv][D] -> [L][Hq][D]."""
    L, Hq, D = Q.shape
    G = Hq // K.shape[1]
    pos = np.arange(L) + first_pos
    q = rot_complex(Q, pos, base)
    k = np.repeat(rot_complex(K, pos, base), G, axis=1)
    v = np.repeat(V, G, axis=1)
    s = np.einsum("ihd,jhd->hij", q, k) / np.sqrt(D)
    s = np.where(np.tril(np.ones((L, L), bool))[None], s, -np.inf)
    p = np.exp(s - logsumexp(s, axis=-1, keepdims=True))
    return np.einsum("hij,jhd->ihd", p, v)


def rand(shape, seed, stream):
    return bf16_bits_to_f64(draw_values_bf16(shape, seed, stream))


def make_case(Lh, Ln, Hq, Hkv, D, seed=0):
    L = Lh + Ln
    Q = rand((L, Hq, D), seed, 1)
    K = rand((L, Hkv, D), seed, 2)
    V = rand((L, Hkv, D), seed, 3)
    return Q, K, V


def test_reuse_equals_full_recompute_cfg1():
    """Benchmark config 1: 256 cached tokens + 32 new, 4 MHA heads of 64, fp32 N(0,1), seed 0."""
    rng = np.random.default_rng(0)
    Lh, Ln, H, D = 256, 32, 4, 64
    Q = rng.standard_normal((Lh + Ln, H, D), dtype=np.float32).astype(np.float64)
    K = rng.standard_normal((Lh + Ln, H, D), dtype=np.float32).astype(np.float64)
    V = rng.standard_normal((Lh + Ln, H, D), dtype=np.float32).astype(np.float64)
    want = full_recompute(Q, K, V)[Lh:]
    got = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:], K[Lh:], V[Lh:])
    assert np.max(np.abs(got - want)) <= 1e-12


@pytest.mark.parametrize("Lh,Ln,Hq,Hkv,D,s", [
    (40, 7, 4, 4, 8, 0), (40, 7, 4, 4, 8, 13), (33, 1, 8, 2, 16, 5), (0, 9, 2, 1, 4, 0),
    (17, 5, 6, 3, 32, 17), (64, 16, 4, 1, 64, 31),
])
def test_truncated_reuse_equals_recompute_of_truncated_tokens(Lh, Ln, Hq, Hkv, D, s):
    """Section 3.4: truncating the saved cache and re-embedding positions must equal what token
    truncation + recomputation gives (positions of the kept tokens restart at 0)."""
    Q, K, V = make_case(Lh, Ln, Hq, Hkv, D, seed=Lh * 31 + Ln)
    want = full_recompute(Q[s:], K[s:], V[s:])[Lh - s:]
    got = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:], K[Lh:], V[Lh:], keep_start=s)
    assert got.shape == (Ln, Hq, D)
    assert np.max(np.abs(got - want)) <= 1e-12


def test_matches_library_sdpa_on_prerotated_inputs():
    """Special case that reduces to a library routine: with Q and K rotated beforehand the rest
    is torch's scaled_dot_product_attention with a boolean mask (fp64, CPU)."""
    Lh, Ln, Hq, Hkv, D, s = 50, 12, 4, 2, 16, 9
    Q, K, V = make_case(Lh, Ln, Hq, Hkv, D, seed=5)
    n = Lh - s
    Kt, Vt = K[s:], V[s:]
    Lk = n + Ln
    q = torch.from_numpy(rot_complex(Q[Lh:], n + np.arange(Ln))).permute(1, 0, 2)
    k = torch.from_numpy(np.repeat(rot_complex(Kt, np.arange(Lk)), Hq // Hkv, axis=1)).permute(1, 0, 2)
    v = torch.from_numpy(np.repeat(Vt, Hq // Hkv, axis=1)).permute(1, 0, 2)
    mask = torch.from_numpy(np.arange(Lk)[None, :] <= (n + np.arange(Ln))[:, None])
    want = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask)
    want = want.permute(1, 0, 2).numpy()
    got = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:], K[Lh:], V[Lh:], keep_start=s)
    assert np.max(np.abs(got - want)) <= 1e-12


@pytest.mark.parametrize("shift", [1.0, 977.0, -250.0, 4095.0])
def test_relative_encoding_shift_invariance(shift):
    """Section 3.4 relies on the encoding being relative: numbering the kept tokens 0..Lk-1, or by
    their original absolute positions s..s+Lk-1, or with any other common offset, is the same."""
    Lh, Ln, Hq, Hkv, D, s = 60, 10, 4, 2, 32, 21
    Q, K, V = make_case(Lh, Ln, Hq, Hkv, D, seed=8)
    a = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:], K[Lh:], V[Lh:], keep_start=s)
    b = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:], K[Lh:], V[Lh:], keep_start=s, pos_shift=shift)
    c = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:], K[Lh:], V[Lh:], keep_start=s, pos_shift=float(s))
    assert np.max(np.abs(a - b)) <= 1e-9
    assert np.max(np.abs(a - c)) <= 1e-9


def test_softmax_rows_and_mask_and_hull():
    Lh, Ln, Hq, Hkv, D, s = 30, 8, 4, 2, 16, 3
    Q, K, V = make_case(Lh, Ln, Hq, Hkv, D, seed=11)
    O, P = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:], K[Lh:], V[Lh:], keep_start=s,
                                   return_probs=True)
    n, Lk = Lh - s, Lh - s + Ln
    assert P.shape == (Hq, Ln, Lk)
    assert np.max(np.abs(P.sum(-1) - 1.0)) <= 1e-14
    assert np.all(P >= 0)
    for j in range(Ln):
        assert np.all(P[:, j, n + j + 1:] == 0.0)      # the future is masked exactly
        assert np.all(P[:, j, :n + j + 1] > 0.0)
    Vt = np.repeat(V[s:], Hq // Hkv, axis=1)
    for j in range(Ln):
        vis = Vt[:n + j + 1]
        assert np.all(O[j] <= vis.max(0) + 1e-12) and np.all(O[j] >= vis.min(0) - 1e-12)
    # O really is P V
    assert np.max(np.abs(np.einsum("hjt,thd->jhd", P, Vt) - O)) <= 1e-13


def test_trivial_special_cases():
    D, H = 8, 2
    Q, K, V = make_case(0, 1, H, H, D, seed=2)
    o = oracle.cached_attention(K[:0], V[:0], Q, K, V)
    assert np.array_equal(o, V)                              # one token sees only itself
    # all keys zero -> uniform weights -> running mean of the visible values
    Lh, Ln = 12, 5
    Q, K, V = make_case(Lh, Ln, H, H, D, seed=3)
    o = oracle.cached_attention(0 * K[:Lh], V[:Lh], Q[Lh:], 0 * K[Lh:], V[Lh:], keep_start=4)
    Vt = V[4:]
    for j in range(Ln):
        assert np.max(np.abs(o[j] - Vt[:Lh - 4 + j + 1].mean(0))) <= 1e-13
    # constant values -> that constant
    Vc = np.broadcast_to(np.linspace(-1, 1, D), V.shape).copy()
    o = oracle.cached_attention(K[:Lh], Vc[:Lh], Q[Lh:], K[Lh:], Vc[Lh:])
    assert np.max(np.abs(o - Vc[Lh:])) <= 1e-13


def test_gqa_equals_mha_with_replicated_kv_heads():
    Lh, Ln, Hq, Hkv, D = 25, 6, 8, 2, 16
    Q, K, V = make_case(Lh, Ln, Hq, Hkv, D, seed=4)
    a = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:], K[Lh:], V[Lh:], keep_start=2)
    Kr, Vr = np.repeat(K, 4, axis=1), np.repeat(V, 4, axis=1)   # consecutive q heads share a kv head
    b = oracle.cached_attention(Kr[:Lh], Vr[:Lh], Q[Lh:], Kr[Lh:], Vr[Lh:], keep_start=2)
    assert np.array_equal(a, b)


def test_scale_is_an_argument_and_defaults_to_inv_sqrt_d():
    Lh, Ln, H, D = 10, 3, 2, 16
    Q, K, V = make_case(Lh, Ln, H, H, D, seed=6)
    a = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:], K[Lh:], V[Lh:])
    b = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:], K[Lh:], V[Lh:], scale=0.25)
    c = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:] * 2.0, K[Lh:], V[Lh:], scale=0.125)
    assert np.max(np.abs(a - b)) <= 1e-15
    assert np.max(np.abs(a - c)) <= 1e-12


def test_naive_kv_truncation_is_wrong():
    """Negative control (Section 4.4, the NKVT baseline): keys cached WITH their old positions,
    truncated, and used beside new tokens numbered in the truncated context give a different
    result, far outside any bf16 tolerance.  Guards against a rebase that silently does nothing."""
    Lh, Ln, Hq, Hkv, D, s = 96, 16, 4, 4, 64, 40
    Q, K, V = make_case(Lh, Ln, Hq, Hkv, D, seed=9)
    good = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:], K[Lh:], V[Lh:], keep_start=s)
    n = Lh - s
    Kt = np.concatenate([K[s:Lh], K[Lh:]]); Vt = np.concatenate([V[s:Lh], V[Lh:]])
    kpos = np.concatenate([np.arange(s, Lh), n + np.arange(Ln)]).astype(np.float64)  # stale history
    qpos = (n + np.arange(Ln)).astype(np.float64)
    bad = oracle.attention_positions(Kt, Vt, Q[Lh:], kpos, qpos, n)
    assert np.max(np.abs(good - bad)) > 0.1
    # with consistent (old, absolute) numbering for everything it is fine again
    ok = oracle.attention_positions(Kt, Vt, Q[Lh:], np.arange(s, Lh + Ln, dtype=np.float64),
                                    np.arange(Lh, Lh + Ln, dtype=np.float64), n)
    assert np.max(np.abs(good - ok)) <= 1e-9


def test_interleaved_style_is_half_split_on_permuted_dims():
    Lh, Ln, H, D = 14, 4, 2, 8
    Q, K, V = make_case(Lh, Ln, H, H, D, seed=12)
    perm = np.empty(D, int)                 # interleaved index 2i -> i, 2i+1 -> i + D/2
    perm[0::2] = np.arange(D // 2); perm[1::2] = np.arange(D // 2) + D // 2
    a = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:], K[Lh:], V[Lh:], keep_start=3, style=0)
    b = oracle.cached_attention(K[:Lh][..., perm], V[:Lh], Q[Lh:][..., perm], K[Lh:][..., perm], V[Lh:],
                                keep_start=3, style=1)
    assert np.max(np.abs(a - b)) <= 1e-13
    # and the two conventions really differ on the same raw data
    c = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:], K[Lh:], V[Lh:], keep_start=3, style=1)
    assert np.max(np.abs(a - c)) > 1e-3


def test_rejects_bad_arguments():
    Q, K, V = make_case(4, 2, 2, 2, 4, seed=1)
    with pytest.raises(ValueError):
        oracle.cached_attention(K[:4], V[:4], Q[4:], K[4:], V[4:], keep_start=5)
    with pytest.raises(ValueError):
        oracle.cached_attention(K[:4], V[:4], Q[4:], K[4:], V[4:], keep_start=-1)


# ---- token discarding lists (Section 3.4, last paragraph) ------------------------------------------------

@pytest.mark.parametrize("kept_kind", ["suffix", "sinks+recent", "scattered", "nothing"])
def test_pruned_history_equals_recompute_over_the_kept_tokens(kept_kind):
    """A discarding list leaves an arbitrary subsequence of the saved tokens; reuse over it must equal
    what a recomputing engine produces on the token sequence [kept history | new turn] at dense
    positions -- and, for a kept suffix, the keep_start path."""
    Lh, Ln, Hq, Hkv, D = 90, 14, 4, 2, 64
    Q, K, V = make_case(Lh, Ln, Hq, Hkv, D, seed=5)
    kept = {"suffix": np.arange(37, Lh), "sinks+recent": np.r_[0:4, 60:Lh],
            "scattered": np.array(sorted(np.random.default_rng(3).choice(Lh, 41, replace=False))),
            "nothing": np.zeros(0, np.int64)}[kept_kind]
    got = oracle.cached_attention_kept(K[:Lh], V[:Lh], kept, Q[Lh:], K[Lh:], V[Lh:])
    seq = np.r_[kept, np.arange(Lh, Lh + Ln)]
    # queries of the history rows do not matter for the new rows; take any (here: the saved ones)
    want = full_recompute(Q[seq], K[seq], V[seq])[len(kept):]
    assert np.abs(got - want).max() < 1e-12
    if kept_kind == "suffix":
        same = oracle.cached_attention(K[:Lh], V[:Lh], Q[Lh:], K[Lh:], V[Lh:], keep_start=37)
        assert np.array_equal(got, same)
    if kept_kind == "scattered":      # dropping different tokens must change the result
        other = oracle.cached_attention_kept(K[:Lh], V[:Lh], np.arange(Lh - 41, Lh), Q[Lh:], K[Lh:], V[Lh:])
        assert np.abs(got - other).max() > 1e-3


def test_compacted_store_gives_what_the_discarding_list_gave():
    """Dropping the discarded rows from the store and then reusing everything that is left is the reuse over the
    pruned history (which is pinned to a full recompute above); hand-checked rows, the empty list and the identity."""
    Lh, Ln, Hq, Hkv, D = 70, 9, 4, 2, 64
    Q, K, V = make_case(Lh, Ln, Hq, Hkv, D, seed=8)
    ranges = [(0, 3), (10, 11), (40, 70)]
    kept = np.r_[0:3, 10:11, 40:70]
    Kc, Vc = oracle.compact_tier(K[:Lh], ranges), oracle.compact_tier(V[:Lh], ranges)
    assert Kc.shape[0] == 34 and np.array_equal(Kc[3], K[10]) and np.array_equal(Kc[4], K[40]) and np.array_equal(Vc[-1], V[69])
    got = oracle.cached_attention(Kc, Vc, Q[Lh:], K[Lh:], V[Lh:], keep_start=0)
    want = oracle.cached_attention_kept(K[:Lh], V[:Lh], kept, Q[Lh:], K[Lh:], V[Lh:])
    assert np.array_equal(got, want)
    assert oracle.compact_tier(K[:Lh], []).shape == (0,) + K.shape[1:]
    assert np.array_equal(oracle.compact_tier(K[:Lh], [(0, Lh)]), K[:Lh])
    # a planted mistake (one range taken one row too early) is seen
    assert not np.array_equal(oracle.compact_tier(K[:Lh], [(0, 3), (9, 10), (40, 70)]), Kc)


def test_sink_discarding_list_closed_forms():
    """Budget arithmetic of the sink-sparing list against hand-computed cases (window 4096, ratio 0.5:
    2048 tokens of [history | new] survive an overflow, as in Section 4.1's 4K/2K setting)."""
    W = 4096
    k = oracle.kept_indices_sinks([3000, 4000, 4000, 5000, 10, 4090, 0], [1000, 100, 2048, 3000, 4000, 7, 50], W, 0.5, 4)
    assert np.array_equal(k[0], np.arange(3000))                                  # 4000 <= 4096: no overflow
    assert np.array_equal(k[1], np.r_[0:4, 4000 - 1944:4000]) and len(k[1]) == 1948   # 2048 - 100 kept
    assert len(k[2]) == 0 and len(k[3]) == 0                                      # the new turn fills the budget
    assert np.array_equal(k[4], np.arange(10))                                    # 4010 <= 4096
    assert np.array_equal(k[5], np.r_[0:4, 4090 - 2037:4090])                     # 2041 kept
    assert len(k[6]) == 0
    # more sinks than budget: only sinks; zero sinks: the plain keep-recent rule of policy 0
    k = oracle.kept_indices_sinks([4000], [2040], W, 0.5, 64)
    assert np.array_equal(k[0], np.arange(8))
    h, n = np.array([4000, 6000, 100]), np.array([500, 100, 30])
    k0 = oracle.kept_indices_sinks(h, n, W, 0.5, 0)
    s0 = oracle.truncate_plan(h, n, W, 0.5, 0)
    for c in range(3):
        assert np.array_equal(k0[c], np.arange(s0[c], h[c]))
