"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, validates configurations and batches, and its truncation planner agrees with
the oracle's bit for bit.  No compute entry point is called here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2403_19708_amd as ca
from paper_2403_19708_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ca.lib_path()):
        from paper_2403_19708_amd import build
        build.build(verbose=False)
    return ca.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ca.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ca_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.SYMBOLS) == names          # the binding covers the whole header


def test_status_strings(lib):
    for code, name in binding.STATUS.items():
        assert lib.ca_status_string(code).decode() == name


def test_config_default_and_struct_layout(lib):
    c = binding._CConfig()
    lib.ca_config_default(ctypes.byref(c))
    assert (c.page_size, c.head_dim, c.rope_style, c.pipeline_depth) == (16, 128, 0, 2)
    assert abs(c.rope_base - 10000.0) < 1e-3 and c.require_load == 1
    ca.config_validate(ca.Config())


@pytest.mark.parametrize("kw,status", [
    (dict(head_dim=96), "CA_ERR_UNSUPPORTED"),
    (dict(page_size=32), "CA_ERR_UNSUPPORTED"),
    (dict(rope_style=2), "CA_ERR_UNSUPPORTED"),
    (dict(n_q_heads=6, n_kv_heads=4), "CA_ERR_INVALID_ARG"),
    (dict(n_layers=0), "CA_ERR_INVALID_ARG"),
    (dict(rope_base=0.5), "CA_ERR_INVALID_ARG"),
    (dict(pipeline_depth=0), "CA_ERR_OUT_OF_RANGE"),
    (dict(max_positions=0), "CA_ERR_OUT_OF_RANGE"),
    (dict(max_batch_q_tokens=1 << 20, max_batch_kv_tokens=1 << 10), "CA_ERR_OUT_OF_RANGE"),
    (dict(attn_variant=7), "CA_ERR_INVALID_ARG"),
    (dict(attn_split=2), "CA_ERR_INVALID_ARG"),
    (dict(attn_prerotate=3), "CA_ERR_INVALID_ARG"),
    (dict(attn_variant=3), "CA_ERR_UNSUPPORTED"),
    (dict(attn_variant=5), "CA_ERR_INVALID_ARG"),
])
def test_config_validation(lib, kw, status):
    with pytest.raises(ca.CaError) as e:
        ca.config_validate(ca.Config(**kw))
    assert e.value.status_name == status


def _good_batch():
    hist = np.array([40, 0, 100], np.int32)
    keep = np.array([8, 0, 100], np.int32)
    new = np.array([5, 17, 3], np.int32)
    bt = np.array([[3, 7, 1, 0], [2, 9, 0, 0], [4, 0, 0, 0]], np.int32)   # needs 3, 2, 1 pages
    return hist, keep, new, bt, 10


def test_batch_validation_accepts_a_good_batch(lib):
    ca.batch_validate(ca.Config(max_positions=128), *_good_batch())


@pytest.mark.parametrize("mutate,status", [
    (lambda h, k, n, bt, p: (h, np.array([41, 0, 100], np.int32), n, bt, p), "CA_ERR_OUT_OF_RANGE"),   # keep_start > hist
    (lambda h, k, n, bt, p: (h, np.array([-1, 0, 100], np.int32), n, bt, p), "CA_ERR_OUT_OF_RANGE"),
    (lambda h, k, n, bt, p: (h, k, np.array([5, 0, 3], np.int32), bt, p), "CA_ERR_INVALID_ARG"),      # empty turn
    (lambda h, k, n, bt, p: (h, k, n, np.where(bt == 9, 10, bt).astype(np.int32), p), "CA_ERR_OUT_OF_RANGE"),  # page id
    (lambda h, k, n, bt, p: (h, k, n, np.where(bt == 9, -1, bt).astype(np.int32), p), "CA_ERR_OUT_OF_RANGE"),
    (lambda h, k, n, bt, p: (h, k, n, np.where(bt == 9, 3, bt).astype(np.int32), p), "CA_ERR_INVALID_ARG"),    # shared page
    (lambda h, k, n, bt, p: (h, k, n, bt[:, :2].copy(), p), "CA_ERR_OUT_OF_RANGE"),                   # too few columns
    (lambda h, k, n, bt, p: (np.array([400, 0, 100], np.int32), k, n, bt, p), "CA_ERR_OUT_OF_RANGE"),  # beyond window
])
def test_batch_validation_rejects(lib, mutate, status):
    with pytest.raises(ca.CaError) as e:
        ca.batch_validate(ca.Config(max_positions=128), *mutate(*_good_batch()))
    assert e.value.status_name == status


def test_batch_validation_limits(lib):
    h, k, n, bt, p = _good_batch()
    with pytest.raises(ca.CaError) as e:
        ca.batch_validate(ca.Config(max_positions=128, max_seqs=2), h, k, n, bt, p)
    assert e.value.status_name == "CA_ERR_OUT_OF_RANGE"
    with pytest.raises(ca.CaError) as e:
        ca.batch_validate(ca.Config(max_positions=128, max_batch_kv_tokens=40, max_batch_q_tokens=30), h, k, n, bt, p)
    assert e.value.status_name == "CA_ERR_OUT_OF_RANGE"


@pytest.mark.parametrize("policy", [0, 1, 2])
def test_planner_agrees_with_oracle_bit_for_bit(lib, policy):
    rng = np.random.default_rng(100 + policy)
    for W, r in ((4096, 0.5), (2048, 0.5), (97, 0.3), (64, 0.75), (4096, 0.1)):
        h = rng.integers(0, 3 * W, 500).astype(np.int32)
        n = rng.integers(0, W, 500).astype(np.int32)
        assert np.array_equal(ca.truncate_plan(h, n, W, r, policy), oracle.truncate_plan(h, n, W, r, policy))


def test_planner_rejects_bad_arguments(lib):
    for kw in (dict(window=0), dict(ratio=0.0), dict(ratio=1.0), dict(policy=3)):
        args = dict(window=16, ratio=0.5, policy=0)
        args.update(kw)
        with pytest.raises(ca.CaError):
            ca.truncate_plan([10], [10], **args)
    with pytest.raises(ca.CaError):
        ca.truncate_plan([-1], [10], 16)


def test_create_without_gpu_fails_cleanly(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(ca.CaError) as e:
        ca.Context(ca.Config())
    assert e.value.status_name in ("CA_ERR_HIP", "CA_ERR_OUT_OF_RANGE")


def _ranges_to_indices(ranges):
    return np.concatenate([np.arange(b, e) for b, e in ranges]) if ranges else np.zeros(0, np.int64)


def test_sink_planner_agrees_with_oracle(lib):
    rng = np.random.default_rng(7)
    for W, r, sink in ((4096, 0.5, 4), (4096, 0.5, 0), (512, 0.25, 16), (97, 0.3, 200), (64, 0.75, 1)):
        h = rng.integers(0, 3 * W, 300).astype(np.int32)
        n = rng.integers(0, W, 300).astype(np.int32)
        got = ca.truncate_plan_sinks(h, n, W, r, sink)
        want = oracle.kept_indices_sinks(h, n, W, r, sink)
        for c in range(300):
            assert len(got[c]) <= 2
            assert np.array_equal(_ranges_to_indices(got[c]), want[c]), (W, r, sink, c)
            assert all(b < e for b, e in got[c]) and (len(got[c]) < 2 or got[c][0][1] < got[c][1][0])


def test_batch_validation_of_kept_ranges(lib):
    h, k, n, bt, p = _good_batch()                  # hist 40, 0, 100; new 5, 17, 3
    cfg = ca.Config(max_positions=128)
    ca.batch_validate(cfg, h, None, n, bt, p, keep_ranges=[[(0, 4), (20, 40)], [], [(3, 9), (9, 10), (50, 55)]])
    for bad, status in (
            ([[(0, 4), (3, 40)], [], []], "CA_ERR_OUT_OF_RANGE"),          # overlap
            ([[(10, 4)], [], []], "CA_ERR_OUT_OF_RANGE"),                  # empty / reversed
            ([[(0, 41)], [], []], "CA_ERR_OUT_OF_RANGE"),                  # beyond hist_len
            ([[(20, 40), (0, 4)], [], []], "CA_ERR_OUT_OF_RANGE"),         # not increasing
            ([[], [(0, 1)], []], "CA_ERR_OUT_OF_RANGE"),                   # hist_len 0 has nothing to keep
            ([[(0, 40)], [], [(0, 100)]], "CA_ERR_OUT_OF_RANGE")):         # 100 + 3 tokens need 7 pages, table has 4
        with pytest.raises(ca.CaError) as e:
            ca.batch_validate(cfg, h, None, n, bt, p, keep_ranges=bad)
        assert e.value.status_name == status, bad
    with pytest.raises(ca.CaError):
        ca.batch_validate(cfg, h, None, n, bt, p)                           # neither keep_start nor ranges


def test_tier_compaction_agrees_with_oracle(lib):
    """ca_tier_compact moves the kept rows of every conversation to the front of its host buffers, in place:
    random range lists (adjacent, touching the ends, empty, everything), and the keep_start form."""
    rng = np.random.default_rng(21)
    row_bytes = 48
    for trial in range(40):
        B = int(rng.integers(1, 6))
        hist = rng.integers(0, 60, B).astype(np.int32)
        K = [rng.integers(0, 256, (int(h), row_bytes), dtype=np.uint8) for h in hist]
        V = [rng.integers(0, 256, (int(h), row_bytes), dtype=np.uint8) for h in hist]
        ranges = []
        for h in hist:
            cuts = np.sort(rng.choice(int(h) + 1, size=min(int(h) + 1, 2 * int(rng.integers(0, 4))), replace=False))
            ranges.append([(int(cuts[i]), int(cuts[i + 1])) for i in range(0, len(cuts) - 1, 2)])
        want_k = [oracle.compact_tier(k, r) for k, r in zip(K, ranges)]
        want_v = [oracle.compact_tier(v, r) for v, r in zip(V, ranges)]
        kb, vb = [k.copy() for k in K], [v.copy() for v in V]
        left = ca.tier_compact(hist, ranges, row_bytes, [k.ctypes.data for k in kb], [v.ctypes.data for v in vb])
        for c in range(B):
            assert left[c] == len(want_k[c]), (trial, c)
            assert np.array_equal(kb[c][:left[c]], want_k[c]) and np.array_equal(vb[c][:left[c]], want_v[c]), (trial, c)
        # the truncation form: one suffix per conversation
        ks = np.array([int(rng.integers(0, h + 1)) for h in hist], dtype=np.int32)
        kb, vb = [k.copy() for k in K], [v.copy() for v in V]
        left = ca.tier_compact(hist, [int(x) for x in ks], row_bytes, [k.ctypes.data for k in kb], [v.ctypes.data for v in vb])
        for c in range(B):
            assert left[c] == hist[c] - ks[c]
            assert np.array_equal(kb[c][:left[c]], K[c][ks[c]:]) and np.array_equal(vb[c][:left[c]], V[c][ks[c]:])


def test_tier_compaction_rejects_bad_ranges_and_moves_nothing(lib):
    rows = np.arange(10 * 8, dtype=np.uint8).reshape(10, 8)
    for bad in ([(0, 4), (3, 6)], [(5, 5)], [(6, 2)], [(0, 11)], [(4, 6), (0, 2)], [(-1, 2)]):
        k, v = rows.copy(), rows.copy()
        with pytest.raises(ca.CaError) as e:
            ca.tier_compact([10], [bad], 8, [k.ctypes.data], [v.ctypes.data])
        assert e.value.status_name == "CA_ERR_OUT_OF_RANGE", bad
        assert np.array_equal(k, rows) and np.array_equal(v, rows)
    # a later conversation's bad range must leave the earlier ones untouched as well
    k0, v0, k1, v1 = rows.copy(), rows.copy(), rows.copy(), rows.copy()
    with pytest.raises(ca.CaError):
        ca.tier_compact([10, 10], [[(2, 4)], [(3, 2)]], 8, [k0.ctypes.data, k1.ctypes.data], [v0.ctypes.data, v1.ctypes.data])
    assert np.array_equal(k0, rows) and np.array_equal(k1, rows)


def test_entry_points_reject_a_null_context_without_touching_a_gpu(lib):
    """Every call that takes a context checks it first: a NULL context is an argument error, not a crash."""
    import ctypes as C
    n = C.c_int64(0)
    ms = C.c_double(0.0)
    assert lib.ca_profile_enable(None, 1) == 1                                           # CA_ERR_INVALID_ARG
    assert lib.ca_profile_read(None, 0, C.byref(ms), C.byref(n)) == 1
    assert lib.ca_profile_timeline(None, None, None, None, 0, C.byref(n)) == 1
    assert lib.ca_sync(None) == 1
    assert lib.ca_join(None, None) == 1
    assert lib.ca_kv_load_layer(None, 0, None, None, None, None) == 1
    assert lib.ca_kv_append_save_layer(None, 0, None, None, None, None, None, None, None) == 1
    assert lib.ca_cached_prefill_attn_static(None, 0, None, None, None, None, C.c_float(1.0), None) == 1
