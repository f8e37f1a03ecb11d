"""Drives the placement manager (include/ca_store.h) with a synthetic multi-turn serving workload and
prints, per eviction policy, where the jobs found their caches.

    python -m paper_2403_19708_amd.store_sim [--sessions 3000] [--mem 40] [--disk 400] ...

Workload recipe (Section 4.1 describes the paper's: ShareGPT conversations, session arrivals Poisson
with rate 1.0 per second; the conversations themselves are replaced by draws here): sessions arrive
as a Poisson process; 27 % have one turn, the rest 2 + geometric turns (mean 5.75 overall); a turn adds
a prompt and an answer of a few hundred tokens, the cache is capped at the context window; the user's
next turn arrives an exponential think time after the previous answer.  One server runs the jobs first
come first served in batches; the jobs that have arrived but not started are the queue the manager
looks ahead into.  Capacities are in units of one full context window of cache.
"""
from __future__ import annotations

import argparse
import heapq
import json

import numpy as np

from . import store as cs


def make_sessions(n, rate, window, rng):
    turns = np.where(rng.random(n) < 0.27, 1, 2 + rng.geometric(1.0 / 5.5, n))
    start = np.cumsum(rng.exponential(1.0 / rate, n))
    out = []
    for s in range(n):
        tokens = rng.integers(40, 900, int(turns[s]))              # prompt + answer of each turn
        out.append(dict(start=float(start[s]), tokens=tokens, think=rng.exponential(60.0, int(turns[s]))))
    return out


def simulate(sessions, policy, prefetch, mem_units, disk_units, buffer_units, window, batch, service, ttl):
    unit = window                                                    # capacity unit: one full window
    st = cs.Store(int(mem_units * unit), int(disk_units * unit), int(buffer_units * unit), policy, prefetch, ttl)
    arrivals = [(s["start"], i, 0) for i, s in enumerate(sessions)]  # (time, session, turn)
    heapq.heapify(arrivals)
    waiting, size, now = [], {}, 0.0
    found = {cs.MISS: 0, cs.HIT_MEM: 0, cs.HIT_DISK: 0}
    first_turns = 0
    try:
        while arrivals or waiting:
            if not waiting:
                now = max(now, arrivals[0][0])
            while arrivals and arrivals[0][0] <= now:
                _, s, t = heapq.heappop(arrivals)
                waiting.append((s, t))
            st.set_queue([s for s, _ in waiting])
            st.prefetch(now)
            running, waiting = waiting[:batch], waiting[batch:]
            st.set_queue([s for s, _ in waiting])
            for s, t in running:
                res = st.lookup(s, now)
                if t == 0:
                    first_turns += 1                                 # nothing could have been stored yet
                else:
                    found[res] += 1
            now += service
            for s, t in running:
                size[s] = min(size.get(s, 0) + int(sessions[s]["tokens"][t]), window)
                st.save(s, size[s], now)
                if t + 1 < len(sessions[s]["tokens"]):
                    heapq.heappush(arrivals, (now + float(sessions[s]["think"][t]), s, t + 1))
            st.take_actions()
        stats = st.stats()
    finally:
        st.close()
    later = sum(found.values())
    return dict(later_turns=later, first_turns=first_turns, hit_memory=found[cs.HIT_MEM] / later,
                hit_disk=found[cs.HIT_DISK] / later, miss=found[cs.MISS] / later,
                fetched=stats["fetched"], evicted=stats["evicted"], dropped=stats["dropped"],
                forced_window_drops=stats["forced_window_drops"])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--sessions", type=int, default=3000)
    ap.add_argument("--rate", type=float, default=1.0, help="new sessions per second")
    ap.add_argument("--window", type=int, default=4096, help="context window in tokens (largest cache of a session)")
    ap.add_argument("--mem", type=float, default=40.0, help="host memory, in full windows")
    ap.add_argument("--disk", type=float, default=400.0, help="disk capacity, in full windows")
    ap.add_argument("--buffer", type=float, default=4.0, help="host memory kept free for fetching, in full windows")
    ap.add_argument("--batch", type=int, default=16)
    ap.add_argument("--service", type=float, default=3.0, help="seconds one batch takes")
    ap.add_argument("--ttl", type=float, default=3600.0)
    ap.add_argument("--seed", type=int, default=0)
    a = ap.parse_args()
    sessions = make_sessions(a.sessions, a.rate, a.window, np.random.default_rng(a.seed))
    out = {}
    for name, policy, prefetch in (("scheduler-aware", cs.SCHEDULER_AWARE, True), ("scheduler-aware, no prefetch", cs.SCHEDULER_AWARE, False),
                                   ("lru", cs.LRU, False), ("fifo", cs.FIFO, False)):
        out[name] = simulate(sessions, policy, prefetch, a.mem, a.disk, a.buffer, a.window, a.batch, a.service, a.ttl)
        r = out[name]
        print(f"{name:30s} memory {r['hit_memory']:.3f}  disk {r['hit_disk']:.3f}  miss {r['miss']:.3f}   "
              f"(fetched {r['fetched']}, evicted {r['evicted']}, dropped {r['dropped']})", flush=True)
    print(json.dumps(dict(config=vars(a), results=out)))


if __name__ == "__main__":
    main()
