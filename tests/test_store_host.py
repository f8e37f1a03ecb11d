"""The library's placement manager (include/ca_store.h) against the oracle, decision by decision: the
same calls go to both, and lookup results, action logs, tier contents, window lengths and counters
must agree exactly.  No GPU is involved (host code of the library only)."""
import os
import re

import numpy as np
import pytest

import paper_2403_19708_amd as ca
from oracle import placement as pl
from paper_2403_19708_amd import store as cs

from test_oracle_placement import read_example

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def lib():
    if not os.path.exists(ca.lib_path()):
        from paper_2403_19708_amd import build
        build.build(verbose=False)
    return ca.load_library()


def test_library_exports_every_symbol_of_the_store_header(lib):
    text = open(os.path.join(ROOT, "include", "ca_store.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(ca_store_[a-z_0-9]+)\s*\(", text)))
    assert len(names) == 14 and sorted(cs.SYMBOLS) == names
    for n in names:
        assert hasattr(lib, n), n
    # the constants of the binding are the header's
    for name, value in re.findall(r"\b(CA_STORE_[A-Z_]+)\s*=\s*(\d+)", text):
        assert getattr(cs, name[len("CA_STORE_"):]) == int(value), name


class Both:
    """feeds the library and the oracle the same calls and compares after each one"""

    def __init__(self, *args, **kw):
        self.lib = cs.Store(*args, **kw)
        self.ref = pl.Store(*args, **kw)

    def close(self):
        self.lib.close()

    def seed(self, session, size, tiers, now=0.0):
        self.lib.seed(session, size, tiers, now)
        it = self.ref.items[session] = pl.Item(size, now, self.ref._next_seq())
        it.in_mem, it.on_disk = bool(tiers & 1), bool(tiers & 2)

    def set_queue(self, q):
        self.lib.set_queue(q)
        self.ref.set_queue(q)

    def prefetch(self, now):
        self.lib.prefetch(now)
        self.ref.prefetch(now)
        self.compare()

    def lookup(self, s, now):
        a, b = self.lib.lookup(s, now), self.ref.lookup(s, now)
        assert a == b, (s, now)
        self.compare()
        return a

    def save(self, s, size, now):
        self.lib.save(s, size, now)
        self.ref.save(s, size, now)
        self.compare()

    def release(self, s, now):
        self.lib.release(s, now)
        self.ref.release(s, now)
        self.compare()

    def compare(self, sessions=None):
        assert self.lib.take_actions() == self.ref.take_actions()
        assert self.lib.windows() == (self.ref.prefetch_window(), self.ref.eviction_window())
        assert self.lib.usage() == (self.ref.mem_used(), self.ref.disk_used(), len(self.ref.items))
        assert self.lib.stats() == self.ref.stats
        for s in (sessions if sessions is not None else list(self.ref.items)):
            assert self.lib.where(s) == self.ref.where(s), s


def test_worked_example_of_the_paper():
    ex = read_example()
    with cs.Store(ex["mem_capacity"][0], ex["disk_capacity"][0], ex["mem_buffer"][0]) as st:
        for s in sorted(set(ex["in_memory"]) | set(ex["on_disk"])):
            st.seed(s, 1, (cs.IN_MEM if s in ex["in_memory"] else 0) | (cs.ON_DISK if s in ex["on_disk"] else 0))
        st.set_queue(ex["queue"])
        assert st.windows() == (ex["prefetch_window"][0], ex["eviction_window"][0])
        st.prefetch(1.0)
        acts = st.take_actions()
        assert [s for k, s in acts if k == cs.FETCH] == ex["fetched"]
        assert [s for k, s in acts if k == cs.EVICT] == ex["evicted_to_disk"]
        assert [s for k, s in acts if k == cs.DROP] == ex["left_the_system"]
        assert len(acts) == 3 and st.take_actions() == []
        everyone = range(1, 11)
        assert [s for s in everyone if st.where(s) & cs.IN_MEM] == ex["memory_after"]
        assert [s for s in everyone if st.where(s) & cs.ON_DISK] == ex["disk_after"]


@pytest.mark.parametrize("policy", [cs.SCHEDULER_AWARE, cs.LRU, cs.FIFO])
@pytest.mark.parametrize("seed", range(6))
def test_random_traces_decision_by_decision(policy, seed):
    rng = np.random.default_rng(31 * seed + policy)
    n_sessions, n_jobs = int(rng.integers(5, 60)), 500
    mem, disk = int(rng.integers(4, 30)), int(rng.integers(0, 60))
    both = Both(mem, disk, int(rng.integers(0, mem // 2 + 1)), policy, prefetch=bool(rng.integers(0, 2)),
                ttl=float(rng.choice([0.0, 25.0, 90.0])))
    try:
        # a state to start from
        for s in range(n_sessions):
            size = int(rng.integers(1, 4))
            tiers = int(rng.integers(0, 4))
            m_used, d_used, _ = both.lib.usage()
            if tiers & 1 and m_used + size > mem:
                tiers &= ~1
            if tiers & 2 and d_used + size > disk:
                tiers &= ~2
            if tiers:
                both.seed(s, size, tiers)
        both.compare()
        jobs = [int(x) for x in rng.integers(0, n_sessions, n_jobs)]
        sizes = {s: int(rng.integers(1, 4)) for s in range(n_sessions)}
        running = []                                           # a small batch of jobs runs at a time
        now = 0.0
        for t, s in enumerate(jobs):
            now += float(rng.exponential(1.0))
            depth = int(rng.integers(0, 15))
            if s in running:
                continue
            both.set_queue(jobs[t:t + depth])
            both.prefetch(now)
            both.set_queue(jobs[t + 1:t + depth])
            both.lookup(s, now)
            running.append(s)
            if len(running) >= int(rng.integers(1, 4)):
                for r in running:
                    now += 0.25
                    if rng.random() < 0.15:                     # the job is abandoned: nothing to write back
                        both.release(r, now)
                        continue
                    sizes[r] = min(sizes[r] + int(rng.integers(0, 2)), min(mem, 6))
                    both.save(r, sizes[r], now)
                running = []
        both.compare(range(n_sessions))
    finally:
        both.close()


def test_argument_errors():
    with pytest.raises(ca.CaError):
        cs.Store(-1, 4)
    with pytest.raises(ca.CaError):
        cs.Store(4, 4, mem_buffer=5)
    with pytest.raises(ca.CaError):
        cs.Store(4, 4, policy=3)
    with cs.Store(4, 4) as st:
        st.seed(1, 2, cs.IN_MEM)
        for bad in (dict(session=1, size=1, tiers=cs.IN_MEM), dict(session=2, size=0, tiers=cs.IN_MEM),
                    dict(session=2, size=1, tiers=0), dict(session=2, size=1, tiers=4)):
            with pytest.raises(ca.CaError) as e:
                st.seed(**bad)
            assert e.value.status_name == "CA_ERR_INVALID_ARG"
        with pytest.raises(ca.CaError) as e:
            st.seed(3, 3, cs.IN_MEM)                            # 2 + 3 > 4
        assert e.value.status_name == "CA_ERR_OUT_OF_RANGE"
        with pytest.raises(ca.CaError) as e:
            st.save(5, 9, 0.0)
        assert e.value.status_name == "CA_ERR_OUT_OF_RANGE" and "exceeds" in str(e.value)
        with pytest.raises(ca.CaError):
            st.save(5, 0, 0.0)
        assert st.usage() == (2, 0, 1) and st.lookup(7, 0.0) == cs.MISS


def test_serving_workload_direction():
    """The synthetic serving workload of the package's driver, with the server saturated so that the queue is
    long: fetching ahead turns disk hits into memory hits, and looking ahead keeps more caches in the
    store than recency or arrival order (the direction of the hit-rate comparison of Section 4.5)."""
    from paper_2403_19708_amd import store_sim
    sessions = store_sim.make_sessions(2000, 1.0, 4096, np.random.default_rng(0))
    run = lambda policy, prefetch: store_sim.simulate(sessions, policy, prefetch, 10, 30, 1, 4096, 16, 3.2, 3600.0)
    aware, plain, lru, fifo = run(cs.SCHEDULER_AWARE, True), run(cs.SCHEDULER_AWARE, False), run(cs.LRU, False), run(cs.FIFO, False)
    for r in (aware, plain, lru, fifo):
        assert abs(r["hit_memory"] + r["hit_disk"] + r["miss"] - 1.0) < 1e-12
    assert aware["hit_disk"] < 0.02 and aware["hit_memory"] > plain["hit_memory"] + 0.1
    assert aware["miss"] < lru["miss"] - 0.05 and aware["miss"] < fifo["miss"] - 0.05
