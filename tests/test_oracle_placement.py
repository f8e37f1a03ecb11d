"""Pins of the placement oracle (Section 3.3) against things other than itself: the worked example the
paper tells, textbook caches written out independently here, the optimal replacement found by brute
force on tiny traces, closed forms of the two window lengths, and invariants on random traces."""
import collections
import itertools
import os

import numpy as np
import pytest

from oracle import placement as pl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "placement_example.txt")


def read_example():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        out[key] = [int(v) for v in vals]
    return out


def seed_store(st, in_memory, on_disk, size=1, now=0.0):
    """puts sessions into a tier directly (a state to start an example from)"""
    for s in sorted(set(in_memory) | set(on_disk)):
        it = st.items[s] = pl.Item(size, now, st._next_seq())
        it.in_mem, it.on_disk = s in in_memory, s in on_disk


def test_worked_example_of_the_paper():
    ex = read_example()
    st = pl.Store(ex["mem_capacity"][0], ex["disk_capacity"][0], ex["mem_buffer"][0], pl.SCHEDULER_AWARE)
    seed_store(st, ex["in_memory"], ex["on_disk"])
    st.set_queue(ex["queue"])
    assert st.prefetch_window() == ex["prefetch_window"][0]
    assert st.eviction_window() == ex["eviction_window"][0]
    st.prefetch(now=1.0)
    acts = st.take_actions()
    assert [s for k, s in acts if k == pl.FETCH] == ex["fetched"]
    assert [s for k, s in acts if k == pl.EVICT] == ex["evicted_to_disk"]
    assert [s for k, s in acts if k == pl.DROP] == ex["left_the_system"]
    assert len(acts) == 3
    assert sorted(s for s in st.items if st.items[s].in_mem) == ex["memory_after"]
    assert sorted(s for s in st.items if st.items[s].on_disk) == ex["disk_after"]
    assert st.stats["forced_window_drops"] == 0


def test_window_lengths_closed_form():
    # C_mem = 10 - 2 = 8, sizes 2, 2, 4 -> S_kv = 8/3; L_pw = floor(8 / (8/3)) = 3; (8 + 12) / (8/3) = 7.5 -> 7
    st = pl.Store(10, 12, 2)
    for s, size in ((1, 2), (2, 2), (3, 4)):
        st.save(s, size, now=0.0)
    assert st.s_kv() == pytest.approx(8 / 3)
    assert st.prefetch_window() == 3 and st.eviction_window() == 7
    # an empty store has nothing to look ahead for
    assert pl.Store(10, 12, 2).prefetch_window() == 0


def run_single_tier(policy, trace, capacity):
    """the memory tier alone (no disks, no buffer, no prefetch), one-unit items; returns hit flags"""
    st = pl.Store(capacity, 0, 0, policy, prefetch=False)
    hits = []
    for t, s in enumerate(trace):
        st.set_queue(trace[t + 1:])
        hits.append(st.lookup(s, now=float(t)) != pl.MISS)
        st.save(s, 1, now=float(t))
    return hits


def textbook_lru(trace, capacity):
    cache, hits = collections.OrderedDict(), []
    for s in trace:
        hits.append(s in cache)
        if s in cache:
            cache.move_to_end(s)
        else:
            if len(cache) == capacity:
                cache.popitem(last=False)
            cache[s] = True
    return hits


def textbook_fifo(trace, capacity):
    order, inside, hits = collections.deque(), set(), []
    for s in trace:
        hits.append(s in inside)
        if s not in inside:
            if len(inside) == capacity:
                inside.discard(order.popleft())
            order.append(s)
            inside.add(s)
    return hits


@pytest.mark.parametrize("seed", range(6))
def test_lru_and_fifo_reduce_to_the_textbook_caches(seed):
    rng = np.random.default_rng(seed)
    trace = [int(x) for x in rng.zipf(1.4, 300) % 23]
    for cap in (1, 3, 8):
        assert run_single_tier(pl.LRU, trace, cap) == textbook_lru(trace, cap)
        assert run_single_tier(pl.FIFO, trace, cap) == textbook_fifo(trace, cap)


def test_a_job_that_ends_without_saving_releases_its_session():
    # textbook LRU in which some accesses are read-only and abandoned: a hit still counts as a use, a miss
    # inserts nothing; written out here, independent of the oracle
    rng = np.random.default_rng(11)
    trace = [int(x) for x in rng.zipf(1.4, 400) % 17]
    aborted = [bool(x) for x in rng.random(400) < 0.3]
    for cap in (1, 3, 6):
        cache, want = collections.OrderedDict(), []
        for s, ab in zip(trace, aborted):
            want.append(s in cache)
            if s in cache:
                cache.move_to_end(s)
            elif not ab:
                if len(cache) == cap:
                    cache.popitem(last=False)
                cache[s] = True
        st = pl.Store(cap, 0, 0, pl.LRU, prefetch=False)
        got = []
        for t, (s, ab) in enumerate(zip(trace, aborted)):
            got.append(st.lookup(s, now=float(t)) != pl.MISS)
            if ab:
                st.release(s, now=float(t))
            else:
                st.save(s, 1, now=float(t))
        assert got == want
        assert not any(i.pinned for i in st.items.values())
    # a session that was looked up and never saved nor released can never leave memory; released, it can
    st = pl.Store(2, 0, 0, pl.LRU, prefetch=False)
    st.save(1, 1, now=0.0); st.save(2, 1, now=1.0)
    assert st.lookup(1, now=2.0) == pl.HIT_MEM
    st.save(3, 1, now=3.0)                      # 1 is pinned: 2 has to go although 1 is older
    assert st.where(1) == 1 and st.where(2) == 0  # bit 0: in memory
    st.release(1, now=4.0)
    st.save(4, 1, now=5.0); st.save(5, 1, now=6.0)
    assert st.where(1) == 0
    st.release(99, now=7.0)                     # unknown session: nothing happens


def fewest_misses(trace, capacity):
    """optimal demand replacement by exhaustive search over every choice of victim"""
    best = [len(trace)]

    def go(t, cache, misses):
        if misses >= best[0]:
            return
        if t == len(trace):
            best[0] = misses
            return
        s = trace[t]
        if s in cache:
            go(t + 1, cache, misses)
        elif len(cache) < capacity:
            go(t + 1, cache | {s}, misses + 1)
        else:
            for v in cache:
                go(t + 1, (cache - {v}) | {s}, misses + 1)
    go(0, frozenset(), 0)
    return best[0]


@pytest.mark.parametrize("seed", range(8))
def test_full_look_ahead_is_the_optimal_replacement(seed):
    """With the whole future in the queue, tail-first eviction is furthest-in-future replacement, whose
    miss count no replacement policy beats; a head-first or recency-based slip shows up as extra misses."""
    rng = np.random.default_rng(100 + seed)
    trace = [int(x) for x in rng.integers(0, 5, 11)]
    for cap in (2, 3):
        hits = run_single_tier(pl.SCHEDULER_AWARE, trace, cap)
        assert hits.count(False) == fewest_misses(trace, cap), (trace, cap)
        assert hits.count(False) <= textbook_lru(trace, cap).count(False)


def test_prefetch_turns_disk_hits_into_memory_hits():
    """Three one-unit sessions on disk, memory of three slots, one kept free as the buffer: jobs inside the
    window of two find their cache in memory; without the fetching scheme each start is a disk hit."""
    for prefetch, want in ((True, [pl.HIT_MEM] * 3), (False, [pl.HIT_DISK] * 3)):
        st = pl.Store(3, 8, 1, pl.SCHEDULER_AWARE, prefetch=prefetch)
        seed_store(st, [], [10, 11, 12])
        queue = [10, 11, 12]
        got = []
        for t in range(3):
            st.set_queue(queue[t:])
            st.prefetch(now=float(t))
            st.set_queue(queue[t + 1:])
            got.append(st.lookup(queue[t], now=float(t)))
            st.save(queue[t], 1, now=float(t) + 0.5)
        assert got == want, prefetch


def test_fetch_does_not_push_out_what_is_needed_sooner():
    # memory: two slots, both taken by the next two jobs; the third job's cache is on disk and stays there
    st = pl.Store(2, 4, 0)
    seed_store(st, [1, 2], [3])
    st.set_queue([1, 2, 3])
    assert st.prefetch_window() == 2
    st.set_queue([1, 3, 2])                      # now 3 is inside the window, but only 2 could make room: it comes later
    st.prefetch(now=0.0)
    assert [k for k, _ in st.take_actions()] == [pl.EVICT, pl.FETCH] and st.where(3) & 1 and st.where(2) == 2
    st = pl.Store(2, 4, 0)
    seed_store(st, [1, 2], [3])
    st.set_queue([2, 3, 1])                      # making room for 3 would cost 1 or 2 ... 1 comes later than 3: it goes
    st.prefetch(now=0.0)
    assert st.where(1) == 2 and st.where(3) & 1
    st = pl.Store(2, 4, 0)
    seed_store(st, [1, 2], [3])
    st.set_queue([1, 2, 3, 3])
    st.prefetch(now=0.0)                         # window of two: job 3 is not looked at
    assert st.take_actions() == []


def test_release_costs_no_write_and_save_invalidates_the_disk_copy():
    st = pl.Store(2, 4, 0)
    seed_store(st, [], [1, 2, 3])
    st.set_queue([1, 2])
    st.prefetch(now=0.0)
    assert st.where(1) == 3 and st.where(2) == 3          # fetched: both copies valid
    st.set_queue([3])
    assert st.lookup(3, now=1.0) == pl.HIT_DISK            # demand load: someone has to leave memory
    acts = st.take_actions()
    assert (pl.RELEASE, 1) in acts and st.stats["bytes_to_disk"] == 0
    st.save(3, 2, now=2.0)                                 # grew to two units; the old disk copy is stale
    assert st.where(3) == 1 and st.mem_used() == 2 and st.where(2) == 2


def test_time_to_live():
    st = pl.Store(4, 4, 0, ttl=10.0)
    st.save(1, 1, now=0.0)
    st.save(2, 1, now=6.0)
    assert st.lookup(1, now=9.0) == pl.HIT_MEM             # touched at 9: lives until 19
    st.save(1, 1, now=9.5)
    assert st.lookup(2, now=16.5) == pl.MISS               # last touched at 6: gone after 16
    assert st.lookup(1, now=19.4) == pl.HIT_MEM
    assert (pl.EXPIRE, 2) in st.take_actions()


@pytest.mark.parametrize("policy", [pl.SCHEDULER_AWARE, pl.LRU, pl.FIFO])
@pytest.mark.parametrize("seed", range(4))
def test_invariants_on_random_traces(policy, seed):
    rng = np.random.default_rng(7 * seed + policy)
    n_sessions, n_jobs = 30, 400
    jobs = [int(x) for x in rng.integers(0, n_sessions, n_jobs)]
    sizes = {s: int(rng.integers(1, 5)) for s in range(n_sessions)}
    st = pl.Store(12, 25, 3, policy, prefetch=True, ttl=0.0)
    stored = set()                                          # sessions that must be found (replayed from the actions)
    for t, s in enumerate(jobs):
        look = jobs[t + 1:t + 1 + int(rng.integers(0, 12))]
        st.set_queue([s] + look)
        st.prefetch(now=float(t))
        st.set_queue(look)
        res = st.lookup(s, now=float(t))
        assert (res != pl.MISS) == (s in stored), (t, s)
        assert st.items.get(s) is None or st.items[s].pinned
        sizes[s] = min(sizes[s] + int(rng.integers(0, 2)), 9)
        st.save(s, sizes[s], now=float(t) + 0.5)
        stored.add(s)
        for kind, who in st.take_actions():
            if kind in (pl.DROP, pl.EXPIRE):
                stored.discard(who)
        assert st.mem_used() <= st.mem_capacity and st.disk_used() <= st.disk_capacity
        assert all(i.in_mem or i.on_disk for i in st.items.values())
        assert set(st.items) == stored
    assert st.stats["hit_mem"] + st.stats["hit_disk"] + st.stats["miss"] == n_jobs


def test_look_ahead_beats_history_on_a_queued_workload():
    """Many sessions take turns while the queue is long: knowing who comes next keeps their caches in the
    store; recency and arrival order do not.  (Direction of the hit-rate comparison of Section 4.5.)"""
    rng = np.random.default_rng(5)
    jobs = [int(x) for x in rng.integers(0, 40, 1500)]
    rate = {}
    for policy in (pl.SCHEDULER_AWARE, pl.LRU, pl.FIFO):
        st = pl.Store(6, 10, 1, policy, prefetch=(policy == pl.SCHEDULER_AWARE))
        for t, s in enumerate(jobs):
            st.set_queue(jobs[t:t + 20])
            st.prefetch(now=float(t))
            st.set_queue(jobs[t + 1:t + 20])
            st.lookup(s, now=float(t))
            st.save(s, 1, now=float(t) + 0.5)
        rate[policy] = (st.stats["hit_mem"] + st.stats["hit_disk"]) / len(jobs)
    assert rate[pl.SCHEDULER_AWARE] > rate[pl.LRU] + 0.05 and rate[pl.SCHEDULER_AWARE] > rate[pl.FIFO] + 0.05, rate
