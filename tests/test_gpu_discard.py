"""Token discarding lists (Section 3.4, last paragraph) on the GPU: the kept saved tokens are given
as ranges; the load brings exactly those into the pages, densely renumbered, and the new turn
attends to them.  Checked against the oracle over the pruned history: pool bytes bit for bit,
outputs within the attention tolerance, for a pinned tier (staged copies) and a device tier (read
in place), with ranges that start and end inside pages."""
import numpy as np
import pytest
import torch

import oracle
import paper_2403_19708_amd as ca
from synth import bf16_bits_to_f64, draw_block_table, draw_values_bf16

from harness import P, bits_to_torch, torch_to_bits
from test_gpu_parity import check_contract, check_tight

pytestmark = pytest.mark.gpu


def ranges_to_indices(ranges):
    return np.concatenate([np.arange(b, e) for b, e in ranges]).astype(np.int64) if ranges else np.zeros(0, np.int64)


def scattered_ranges(hist, seed):
    """an importance-pruned history: short runs of kept tokens separated by short gaps"""
    rng = np.random.default_rng(seed)
    out, at = [], int(rng.integers(0, 5))
    while at < hist:
        run = int(rng.integers(1, 9))
        out.append((at, min(hist, at + run)))
        at += run + int(rng.integers(1, 7))
    return out


@pytest.mark.parametrize("tier", ["pinned", "device"])
@pytest.mark.parametrize("kind", ["sinks+recent", "scattered"])
def test_discarding_list_load_and_attention(tier, kind):
    Hq, Hkv, D, W = 8, 2, 128, 512
    hist = np.array([700, 333, 90], np.int32)
    new = np.array([60, 9, 140], np.int32)
    B, seed = len(hist), 83
    if kind == "sinks+recent":
        keep = ca.truncate_plan_sinks(hist, new, W, 0.5, 4)
        want_idx = oracle.kept_indices_sinks(hist, new, W, 0.5, 4)
        assert len(keep[0]) == 2 and len(keep[1]) == 1 and keep[2] == [(0, 90)]     # overflow, no overflow, no overflow
    else:
        keep = [scattered_ranges(int(hist[0]), 1)[:40], scattered_ranges(int(hist[1]), 2), []]
        want_idx = [ranges_to_indices(r) for r in keep]
    for c in range(B):
        assert np.array_equal(ranges_to_indices(keep[c]), want_idx[c])
    n_keep = np.array([len(i) for i in want_idx], np.int32)
    full_k = [draw_values_bf16((int(hist[c] + new[c]), Hkv, D), seed, 10 + c) for c in range(B)]
    full_v = [draw_values_bf16((int(hist[c] + new[c]), Hkv, D), seed, 20 + c) for c in range(B)]
    q_bits = [draw_values_bf16((int(new[c]), Hq, D), seed, 30 + c) for c in range(B)]
    dev = torch.device("cuda:0")
    mk = (lambda a: bits_to_torch(a, pin=True)) if tier == "pinned" else (lambda a: bits_to_torch(a, dev))
    tier_k = [mk(full_k[c][:hist[c]]) for c in range(B)]
    tier_v = [mk(full_v[c][:hist[c]]) for c in range(B)]
    pages = (n_keep + new + P - 1) // P
    num_pages = int(pages.sum()) + 5
    bt = draw_block_table(pages, num_pages, seed)
    sentinel = 0x7FC0
    k_pool = torch.empty((num_pages, Hkv, P, D), dtype=torch.bfloat16, device=dev)
    k_pool.view(torch.int16).fill_(np.array(sentinel, np.uint16).view(np.int16).item())
    v_pool = k_pool.clone()
    take = lambda full: bits_to_torch(np.concatenate([full[c][hist[c]:] for c in range(B)]), dev)
    kn, vn = take(full_k), take(full_v)
    q = bits_to_torch(np.concatenate(q_bits), dev)
    out = torch.zeros_like(q)
    cfg = ca.Config(n_layers=1, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, max_positions=W, max_seqs=B,
                    max_batch_kv_tokens=int((n_keep + new).sum()) + 64, max_batch_q_tokens=int(new.sum()) + 16)
    w = bf16_bits_to_f64
    with ca.Context(cfg) as ctx:
        ctx.rope_rebase(hist, None, new, bt, num_pages, keep_ranges=keep)
        assert np.array_equal(ctx.rebase_read(0), n_keep)
        meta = oracle.rebase(n_keep, np.zeros(B, np.int32), new, bt, P)      # only the kept counts matter to it
        assert np.array_equal(ctx.rebase_read(5), meta["slot_map"]) and np.array_equal(ctx.rebase_read(3), meta["q_pos"])
        ctx.kv_load_layer(0, tier_k, tier_v, k_pool, v_pool)
        ctx.kv_append_layer(0, kn, vn, k_pool, v_pool)
        ctx.cached_prefill_attn(0, q, k_pool, v_pool, out, 1.0 / np.sqrt(D))
        ctx.sync(); torch.cuda.synchronize()
        # pool: kept tokens then the new turn, page by page as the block table says; everything else untouched
        for name, pool, full in (("k", k_pool, full_k), ("v", v_pool, full_v)):
            want = np.full((num_pages, Hkv, P, D), sentinel, np.uint16)
            for c in range(B):
                rows = np.ascontiguousarray(np.concatenate([full[c][want_idx[c]], full[c][hist[c]:]]))
                oracle.unpack(rows, 0, want, bt[c], P, Hkv, D, 0, len(rows))
            assert np.array_equal(torch_to_bits(pool), want), name
        got = torch_to_bits(out)
        at = 0
        for c in range(B):
            ref = oracle.cached_attention_kept(w(full_k[c][:hist[c]]), w(full_v[c][:hist[c]]), want_idx[c], w(q_bits[c]),
                                               w(full_k[c][hist[c]:]), w(full_v[c][hist[c]:]))
            check_contract(w(got[at:at + int(new[c])]), ref, c)
            check_tight(w(got[at:at + int(new[c])]), ref, int(n_keep[c]), c)
            at += int(new[c])


def test_compacted_tier_serves_the_next_turn_like_the_discarding_list():
    """After ca_tier_compact has dropped the discarded rows from the pinned tier, loading everything that is left
    gives the pool bytes and the attention output, bit for bit, that loading the kept ranges of the uncompacted tier
    gave; the compacted tier holds the oracle's rows."""
    Hq, Hkv, D, W = 8, 2, 128, 1024
    hist = np.array([700, 333, 90], np.int32)
    new = np.array([60, 9, 140], np.int32)
    B, seed = len(hist), 85
    keep = [scattered_ranges(int(hist[0]), 5)[:50], [(0, 4), (200, 333)], [(0, 90)]]
    n_keep = np.array([len(ranges_to_indices(r)) for r in keep], np.int32)
    full_k = [draw_values_bf16((int(hist[c] + new[c]), Hkv, D), seed, 10 + c) for c in range(B)]
    full_v = [draw_values_bf16((int(hist[c] + new[c]), Hkv, D), seed, 20 + c) for c in range(B)]
    dev = torch.device("cuda:0")
    tier_k = [bits_to_torch(full_k[c][:hist[c]], pin=True) for c in range(B)]
    tier_v = [bits_to_torch(full_v[c][:hist[c]], pin=True) for c in range(B)]
    pages = (n_keep + new + P - 1) // P
    num_pages = int(pages.sum()) + 5
    bt = draw_block_table(pages, num_pages, seed)
    take = lambda full: bits_to_torch(np.concatenate([full[c][hist[c]:] for c in range(B)]), dev)
    kn, vn = take(full_k), take(full_v)
    q = bits_to_torch(np.concatenate([draw_values_bf16((int(new[c]), Hq, D), seed, 30 + c) for c in range(B)]), dev)
    cfg = ca.Config(n_layers=1, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, max_positions=W, max_seqs=B,
                    max_batch_kv_tokens=int((n_keep + new).sum()) + 64, max_batch_q_tokens=int(new.sum()) + 16)

    def turn(ctx, hist_now, keep_ranges):
        k_pool = torch.zeros((num_pages, Hkv, P, D), dtype=torch.bfloat16, device=dev)
        v_pool = torch.zeros_like(k_pool)
        out = torch.zeros_like(q)
        ctx.rope_rebase(hist_now, None if keep_ranges is not None else np.zeros(B, np.int32), new, bt, num_pages, keep_ranges=keep_ranges)
        ctx.kv_load_layer(0, tier_k, tier_v, k_pool, v_pool)
        ctx.kv_append_layer(0, kn, vn, k_pool, v_pool)
        ctx.cached_prefill_attn(0, q, k_pool, v_pool, out, 1.0 / np.sqrt(D))
        ctx.sync(); torch.cuda.synchronize()
        return torch_to_bits(k_pool).copy(), torch_to_bits(v_pool).copy(), torch_to_bits(out).copy()

    with ca.Context(cfg) as ctx:
        before = turn(ctx, hist, keep)
        left = ca.tier_compact(hist, keep, Hkv * D * 2, tier_k, tier_v)
        assert np.array_equal(left, n_keep)
        for c in range(B):
            assert np.array_equal(torch_to_bits(tier_k[c])[:left[c]], oracle.compact_tier(full_k[c][:hist[c]], keep[c])), c
            assert np.array_equal(torch_to_bits(tier_v[c])[:left[c]], oracle.compact_tier(full_v[c][:hist[c]], keep[c])), c
        after = turn(ctx, left, None)
    for a, b in zip(before, after):
        assert np.array_equal(a, b)
