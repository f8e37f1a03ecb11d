"""Seeded random batches through the whole layer path (rebase, load, append, attention, save) against
the oracle: shapes, lengths, truncation points, head grouping, pair convention and the library's
scheduling switches (key splitting, key pre-rotation, kernel choice, tile size) are all drawn, so that
combinations nobody wrote down by hand get exercised.  Outputs within the attention tolerance, pool
and tier bytes bit for bit."""
import numpy as np
import pytest

import oracle  # noqa: F401  (Case uses it)
from harness import Case, GpuRun, torch_to_bits
from test_gpu_parity import check_contract, check_tight

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(1000 + seed)
    B = int(rng.integers(1, 6))
    Hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 2, 4, 8]))
    D = int(rng.choice([64, 128]))
    style = int(rng.integers(0, 2))
    hist = rng.integers(0, 900, B).astype(np.int32)
    hist[rng.random(B) < 0.2] = 0                                   # some conversations start fresh
    new = np.where(rng.random(B) < 0.3, rng.integers(1, 4, B), rng.integers(1, 300, B)).astype(np.int32)
    keep = np.array([int(rng.integers(0, h + 1)) if rng.random() < 0.6 else 0 for h in hist], np.int32)
    knobs = dict(attn_split=int(rng.integers(0, 2)), attn_prerotate=int(rng.choice([0, 1, 2])), attn_schedule=int(rng.integers(0, 2)),
                 attn_variant=int(rng.choice([0, 0, 2])), attn_tile_rows=int(rng.choice([0, 0, 128, 256])))
    case = Case(hist, new, keep, Hkv * G, Hkv, D, seed=2000 + seed, style=style, window=2048)
    return case, knobs


@pytest.mark.parametrize("seed", range(16))
def test_random_batch_matches_oracle(seed):
    case, knobs = draw_case(seed)
    run = GpuRun(case, tier="pinned" if seed % 2 else "device", **knobs)
    try:
        run.rebase()
        run.run_layer(0)
        run.finish()
        for c in range(case.B):
            check_contract(run.out_f64(0, c), case.oracle_out(0, c), (seed, knobs, c))
            check_tight(run.out_f64(0, c), case.oracle_out(0, c), int(case.n_keep[c]), (seed, knobs, c))
        for which, pool, host in (("k", run.k_pool[0], run.host_k[0]), ("v", run.v_pool[0], run.host_v[0])):
            assert np.array_equal(torch_to_bits(pool), case.oracle_pool(0, which)), (seed, which)
            for c in range(case.B):
                got = torch_to_bits(host[c])
                assert np.array_equal(got[:case.hist_len[c]], case.tensor(0, f"{which}_hist", c)), (seed, which, c)
                assert np.array_equal(got[case.hist_len[c]:], case.tensor(0, f"{which}_new", c)), (seed, which, c)
    finally:
        run.close()


def draw_decode_case(seed):
    """every conversation brings one or two new tokens and the heads are grouped by two at most: the shape the
    streaming decode kernel takes under the automatic choice"""
    rng = np.random.default_rng(5000 + seed)
    B = int(rng.integers(1, 9))
    Hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 1, 2]))
    D = int(rng.choice([64, 128]))
    style = int(rng.integers(0, 2))
    hist = np.where(rng.random(B) < 0.15, 0, rng.integers(0, 3000, B)).astype(np.int32)
    new = rng.integers(1, (2 // G) + 1, B).astype(np.int32)
    keep = np.array([int(rng.integers(0, h + 1)) if rng.random() < 0.4 else 0 for h in hist], np.int32)
    knobs = dict(attn_split=int(rng.integers(0, 2)), attn_variant=int(rng.choice([0, 4, 2])))
    return Case(hist, new, keep, Hkv * G, Hkv, D, seed=6000 + seed, style=style, window=4096), knobs


@pytest.mark.parametrize("seed", range(12))
def test_random_decode_batch_matches_oracle(seed):
    case, knobs = draw_decode_case(seed)
    run = GpuRun(case, tier="device", **knobs)
    try:
        run.rebase()
        run.run_layer(0)
        run.finish()
        for c in range(case.B):
            check_contract(run.out_f64(0, c), case.oracle_out(0, c), (seed, knobs, c))
            check_tight(run.out_f64(0, c), case.oracle_out(0, c), int(case.n_keep[c]), (seed, knobs, c))
        for which, pool in (("k", run.k_pool[0]), ("v", run.v_pool[0])):
            assert np.array_equal(torch_to_bits(pool), case.oracle_pool(0, which)), (seed, which)
    finally:
        run.close()
