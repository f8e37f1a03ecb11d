"""Pins for the oracle's integer/byte work: truncation planner, rebased metadata, pack/unpack and
the KV-size closed form, against values the paper prints, numpy re-formulations and brute force.
CPU only."""
import numpy as np
import pytest

import oracle
from synth import draw_block_table


# ---------------------------------------------------------------- closed forms from the paper
def test_kv_bytes_per_token_matches_printed_values(golden):
    for model in ("llama65b", "llama13b", "llama70b", "falcon40b"):
        layers, kv_heads, dim = (int(x) for x in golden[f"shape.{model}"].split())
        mib = oracle.kv_bytes_per_token(layers, kv_heads, dim, 2) / 2 ** 20
        printed = float(golden[f"kv_mb_per_token.{model}"])
        digits = len(golden[f"kv_mb_per_token.{model}"].split(".")[1])
        assert abs(mib - printed) <= 0.5 * 10 ** (-digits) + 1e-12, (model, mib, printed)


def test_transfer_example_is_consistent(golden):
    layers, kv_heads, dim = (int(x) for x in golden["shape.llama65b"].split())
    tokens = int(golden["load_example.tokens"])
    gib = tokens * oracle.kv_bytes_per_token(layers, kv_heads, dim, 2) / 2 ** 30
    assert gib == float(golden["load_example.kv_gb"])
    load_ms = gib / float(golden["load_example.link_gb_per_s"]) * 1e3
    assert abs(load_ms - float(golden["load_example.load_ms"])) < 0.5
    gen = gib / (float(golden["load_example.prefill_ms"]) / 1e3)
    assert abs(gen - float(golden["load_example.kv_gen_gb_per_s"])) < 0.05
    fill = float(golden["load_example.free_hbm_gb"]) / gen
    assert abs(fill - float(golden["load_example.fill_seconds"])) < 0.5


# ---------------------------------------------------------------- truncation planner
def test_planner_reproduces_the_papers_example(golden):
    W = int(golden["truncation_example.window"])
    cut = int(golden["truncation_example.cut"])
    kept = int(golden["truncation_example.kept_kv"])
    r = float(golden["truncation_example.ratio"])
    # a context that has just overflowed: 3584 saved tokens + 513 new ones (> 4096)
    # "keep the most recent half window": kept history + new = 2048
    s = oracle.truncate_plan([3584], [512 + 1], W, r, policy=0)[0]
    assert 3584 - s == W - cut - 513
    s = oracle.truncate_plan([4000], [512], W, r, policy=0)[0]
    assert 4000 - s == kept
    # "cut off the first 2K tokens": 3584 saved -> KV[0:1536] survives
    s = oracle.truncate_plan([3584], [513], W, r, policy=1)[0]
    assert s == cut and 3584 - s == kept
    # "discard the earliest half of the tokens": 3072 + 1026 = 4098 -> drop 2049
    s = oracle.truncate_plan([3072], [1026], W, r, policy=2)[0]
    assert s == 2049


def test_planner_no_overflow_means_no_truncation():
    h = np.array([0, 10, 4000, 4095, 2048], np.int32)
    n = np.array([5, 10, 96, 1, 2048], np.int32)
    for pol in (0, 1, 2):
        assert np.array_equal(oracle.truncate_plan(h, n, 4096, 0.5, pol), np.zeros(5, np.int32))


@pytest.mark.parametrize("policy", [0, 1, 2])
def test_planner_properties_brute_force(policy):
    rng = np.random.default_rng(policy)
    for W, r in ((64, 0.5), (100, 0.25), (4096, 0.5), (37, 0.7)):
        h = rng.integers(0, 3 * W, 200).astype(np.int32)
        n = rng.integers(1, W // 2 + 1, 200).astype(np.int32)
        s = oracle.truncate_plan(h, n, W, r, policy)
        assert np.all(s >= 0) and np.all(s <= h)
        over = h.astype(int) + n > W
        assert np.all(s[~over] == 0)
        kept = h - s
        assert np.all(kept[over] + n[over] <= W)           # fits again
        for c in np.nonzero(over)[0]:
            if policy == 0:
                want = min(max(int(np.floor(W * (1 - r))) - int(n[c]), 0), int(h[c]))
                assert kept[c] == want
            elif policy == 1:
                drop = int(np.floor(W * r))
                k = 0
                while h[c] - min(k * drop, h[c]) + n[c] > W and k * drop < h[c]:
                    k += 1
                assert s[c] == min(k * drop, h[c])
            else:
                cur = 0
                while h[c] - cur + n[c] > W and cur < h[c]:
                    cur = min(int(h[c]), cur + max(1, int(np.floor(r * (h[c] - cur + n[c])))))
                assert s[c] == cur


def test_planner_rejects_bad_arguments():
    for kw in (dict(window=0), dict(ratio=0.0), dict(ratio=1.0), dict(policy=3)):
        args = dict(window=16, ratio=0.5, policy=0); args.update(kw)
        with pytest.raises(ValueError):
            oracle.truncate_plan([10], [10], **args)


# ---------------------------------------------------------------- rebased metadata
def test_rebase_metadata_against_numpy_formulation():
    rng = np.random.default_rng(3)
    B, P = 7, 16
    h = rng.integers(0, 300, B).astype(np.int32); h[2] = 0
    n = rng.integers(1, 70, B).astype(np.int32)
    s = (rng.random(B) * (h + 1)).astype(np.int32); s[0] = 0; s[1] = h[1]
    lk = h - s + n
    pages = (lk + P - 1) // P
    bt = draw_block_table(pages, int(pages.sum()) + 11, seed=5)
    m = oracle.rebase(h, s, n, bt, P)
    assert np.array_equal(m["n_keep"], h - s)
    assert np.array_equal(m["cu_q"], np.concatenate([[0], np.cumsum(n)]))
    assert np.array_equal(m["cu_k"], np.concatenate([[0], np.cumsum(lk)]))
    assert np.array_equal(m["q_seq"], np.repeat(np.arange(B), n))
    assert np.array_equal(m["q_pos"], np.concatenate([np.arange(a, a + b) for a, b in zip(h - s, n)]))
    t = np.concatenate([np.arange(x) for x in lk]); c = np.repeat(np.arange(B), lk)
    assert np.array_equal(m["slot_map"], bt[c, t // P] * P + t % P)
    # every context token has its own slot
    assert len(np.unique(m["slot_map"])) == int(lk.sum())
    # last query of a conversation sits at the last key position
    for i in range(B):
        assert m["q_pos"][m["cu_q"][i + 1] - 1] == lk[i] - 1


def test_rebase_rejects_bad_arguments():
    bt = np.zeros((1, 2), np.int32)
    with pytest.raises(ValueError):
        oracle.rebase([10], [11], [4], bt, 16)            # keep_start beyond the history
    with pytest.raises(ValueError):
        oracle.rebase([40], [0], [4], bt, 16)             # needs 3 pages, table has 2


# ---------------------------------------------------------------- pack / unpack
def _pool(num_pages, Hkv, P, D, dtype, fill):
    return np.full((num_pages, Hkv, P, D), fill, dtype=dtype)


@pytest.mark.parametrize("dtype", [np.uint16, np.float32, np.uint8])
def test_unpack_matches_fancy_indexing_and_leaves_the_rest_alone(dtype):
    rng = np.random.default_rng(1)
    P, Hkv, D = 16, 3, 8
    hist, s, new = 45, 7, 9                               # source offset 7: not page aligned
    n = hist - s
    lk = n + new
    pages = (lk + P - 1) // P
    bt = draw_block_table([pages], pages + 5, seed=2)[0]
    src = rng.integers(0, 200, (hist, Hkv, D)).astype(dtype)
    sentinel = 251 if dtype != np.float32 else -7.5
    pool = _pool(pages + 5, Hkv, P, D, dtype, sentinel)
    oracle.unpack(src, s, pool, bt, P, Hkv, D, 0, n)
    want = _pool(pages + 5, Hkv, P, D, dtype, sentinel)
    t = np.arange(n)
    want[bt[t // P], :, t % P, :] = src[s + t]
    assert np.array_equal(pool, want)
    # pack reads the same tokens back, into the middle of a larger buffer
    out = np.full((n + 6, Hkv, D), sentinel, dtype=dtype)
    oracle.pack(pool, bt, P, Hkv, D, 0, n, out, 3)
    assert np.array_equal(out[3:3 + n], src[s:])
    assert np.all(out[:3] == sentinel) and np.all(out[3 + n:] == sentinel)


def test_pack_unpack_roundtrip_and_page_permutation_invariance():
    rng = np.random.default_rng(4)
    P, Hkv, D = 16, 2, 4
    lk = 70
    pages = (lk + P - 1) // P
    src = rng.integers(0, 60000, (lk, Hkv, D)).astype(np.uint16)
    outs = []
    for seed in (1, 2):
        bt = draw_block_table([pages], 3 * pages, seed=seed)[0]
        pool = np.zeros((3 * pages, Hkv, P, D), np.uint16)
        oracle.unpack(src, 0, pool, bt, P, Hkv, D, 0, lk)
        back = np.zeros_like(src)
        oracle.pack(pool, bt, P, Hkv, D, 0, lk, back, 0)
        assert np.array_equal(back, src)
        # a sub-range that starts and ends inside pages
        part = np.zeros((31, Hkv, D), np.uint16)
        oracle.pack(pool, bt, P, Hkv, D, 19, 31, part, 0)
        assert np.array_equal(part, src[19:50])
        outs.append(back)
    assert np.array_equal(outs[0], outs[1])


def test_unpack_append_after_history():
    """New-turn tokens are appended behind the kept history in the same paged sequence."""
    rng = np.random.default_rng(6)
    P, Hkv, D = 16, 2, 4
    n, new = 21, 13
    pages = (n + new + P - 1) // P
    bt = draw_block_table([pages], pages + 2, seed=9)[0]
    hist = rng.integers(0, 60000, (n, Hkv, D)).astype(np.uint16)
    fresh = rng.integers(0, 60000, (new, Hkv, D)).astype(np.uint16)
    pool = np.zeros((pages + 2, Hkv, P, D), np.uint16)
    oracle.unpack(hist, 0, pool, bt, P, Hkv, D, 0, n)
    oracle.unpack(fresh, 0, pool, bt, P, Hkv, D, n, new)
    back = np.zeros((n + new, Hkv, D), np.uint16)
    oracle.pack(pool, bt, P, Hkv, D, 0, n + new, back, 0)
    assert np.array_equal(back, np.concatenate([hist, fresh]))
