"""Oracle of the hierarchical KV-cache placement (Section 3.3): which conversation sessions' caches
sit in host memory, which on disk, what is fetched ahead of the job queue and what is evicted.

TEST INFRASTRUCTURE ONLY.  Plain Python over lists and dicts, every decision a linear scan, written
from the section's prose in its order: the look-ahead prefetching window (Section 3.3.1), the
look-ahead eviction window and its tail-first rule (Section 3.3.2), the host-memory buffer, one item
per session as the unit of movement, and the time to live of Section 4.5.  The least-recently-used
and first-in-first-out policies the section compares against run through the same flows with a
different choice of victim.

The section leaves several points open; the readings taken here (the library takes the same ones):

  * S_kv, "the average KV size of a session", is the mean size of the items stored right now.
  * C_mem of both window formulas is the memory capacity minus the reserved buffer.
  * Fetching copies: the disk copy of a fetched item stays valid until the session is saved again
    (the example of Section 3.3.2 needs this: the disks are still full after Job 3 was fetched).
    An item evicted from memory that still has a valid disk copy costs no write.
  * Victim order of the scheduler-aware policy, in memory and on disk alike: sessions with no job in
    the queue first (least recently used among them), then the session whose next job is furthest
    from the head.  Items with a job inside the eviction window are thereby dropped from the system
    only when nothing else is left; such forced drops are counted.
  * When an item leaves memory and the disks are full, the incoming item competes with the disk
    items under the same order and is itself dropped if it ranks last (scheduler-aware only).
  * A fetch never evicts an item whose job comes sooner than the job fetched for.
  * The session of the running job is pinned in memory from lookup to save (or to release, for a job that
    ends without saving).
"""
from __future__ import annotations

SCHEDULER_AWARE, LRU, FIFO = 0, 1, 2
MISS, HIT_MEM, HIT_DISK = 0, 1, 2
# action kinds
FETCH, LOAD, EVICT, RELEASE, DROP_DISK, DROP, EXPIRE = 1, 2, 3, 4, 5, 6, 7


class Item:
    def __init__(self, size, now, seq):
        self.size = size
        self.in_mem = False
        self.on_disk = False
        self.pinned = False
        self.last_access = now
        self.mem_seq = seq      # order of arrival in memory / on disk (first-in-first-out)
        self.disk_seq = seq


class Store:
    def __init__(self, mem_capacity, disk_capacity, mem_buffer=0, policy=SCHEDULER_AWARE, prefetch=True, ttl=0.0):
        assert mem_capacity >= 0 and disk_capacity >= 0 and 0 <= mem_buffer <= mem_capacity
        self.mem_capacity, self.disk_capacity, self.mem_buffer = mem_capacity, disk_capacity, mem_buffer
        self.policy, self.prefetch_on, self.ttl = policy, prefetch, ttl
        self.items = {}
        self.queue = []
        self.actions = []
        self.seq = 0
        self._keep = None
        self.stats = dict(lookups=0, hit_mem=0, hit_disk=0, miss=0, fetched=0, loaded=0, evicted=0, released=0,
                          dropped=0, expired=0, forced_window_drops=0, bytes_to_disk=0, bytes_from_disk=0)

    # ---- bookkeeping ---------------------------------------------------------------------------------
    def mem_used(self):
        return sum(i.size for i in self.items.values() if i.in_mem)

    def disk_used(self):
        return sum(i.size for i in self.items.values() if i.on_disk)

    def where(self, session):
        i = self.items.get(session)
        return (0 if i is None else (1 if i.in_mem else 0) | (2 if i.on_disk else 0))

    def s_kv(self):
        return sum(i.size for i in self.items.values()) / len(self.items) if self.items else 0.0

    def _window(self, capacity):
        """floor(capacity / S_kv) with S_kv = total / count, in whole numbers: floor(capacity * count / total)"""
        total = sum(i.size for i in self.items.values())
        return (capacity * len(self.items)) // total if total > 0 else 0

    def prefetch_window(self):
        """L_pw = C_mem / S_kv (Section 3.3.1)"""
        return self._window(self.mem_capacity - self.mem_buffer)

    def eviction_window(self):
        """(C_mem + C_disk) / S_kv (Section 3.3.2)"""
        return self._window(self.mem_capacity - self.mem_buffer + self.disk_capacity)

    def position(self, session):
        for p, s in enumerate(self.queue):
            if s == session:
                return p
        return None

    def _next_seq(self):
        self.seq += 1
        return self.seq

    def _forget_if_gone(self, session):
        i = self.items[session]
        if not i.in_mem and not i.on_disk:
            del self.items[session]

    # ---- choice of victim ----------------------------------------------------------------------------
    def _rank(self, session, tier):
        """sort key: the smallest key is evicted first"""
        i = self.items[session]
        if self.policy == LRU:
            return (i.last_access, session)
        if self.policy == FIFO:
            return (i.mem_seq if tier == "mem" else i.disk_seq, session)
        p = self.position(session)
        if p is None:
            return (0, i.last_access, session)      # nobody waits for it: oldest access first
        return (1, -p, session)                      # tail of the queue first

    def _victim(self, candidates, tier):
        return min(candidates, key=lambda s: self._rank(s, tier)) if candidates else None

    # ---- movements ---------------------------------------------------------------------------------
    def _drop_disk_copy(self, session):
        i = self.items[session]
        i.on_disk = False
        if i.in_mem:
            self.actions.append((DROP_DISK, session))
        else:
            self.actions.append((DROP, session))
            self.stats["dropped"] += 1
            p = self.position(session)
            if p is not None and p < self.eviction_window():
                self.stats["forced_window_drops"] += 1
        self._forget_if_gone(session)

    def _evict_from_memory(self, session):
        """memory -> disk (Section 3.3.2); the item may end up outside the system when the disks are full"""
        i = self.items[session]
        assert i.in_mem and not i.pinned
        if i.on_disk:                                   # a valid copy is already there
            i.in_mem = False
            self.actions.append((RELEASE, session))
            self.stats["released"] += 1
            return
        while i.size > self.disk_capacity - self.disk_used():
            on_disk = [s for s, it in self.items.items() if it.on_disk and s != self._keep]
            if i.size > self.disk_capacity or not on_disk:
                victim = session
            elif self.policy == SCHEDULER_AWARE:
                victim = self._victim(on_disk + [session], "disk")
            else:
                victim = self._victim(on_disk, "disk")
            if victim == session:                       # the incoming item ranks last: it leaves the system
                i.in_mem = False
                self.actions.append((DROP, session))
                self.stats["dropped"] += 1
                p = self.position(session)
                if p is not None and p < self.eviction_window():
                    self.stats["forced_window_drops"] += 1
                self._forget_if_gone(session)
                return
            self._drop_disk_copy(victim)
        i.in_mem, i.on_disk, i.disk_seq = False, True, self._next_seq()
        self.actions.append((EVICT, session))
        self.stats["evicted"] += 1
        self.stats["bytes_to_disk"] += i.size

    def _make_room(self, need_free, not_sooner_than=None, keep=None):
        """evict from memory until need_free units are free; False if the remaining candidates are all
        pinned, or wanted sooner than queue position not_sooner_than"""
        self._keep = keep                                # being brought in: its disk copy is not a victim either
        ok = True
        while ok and self.mem_capacity - self.mem_used() < need_free:
            cands = [s for s, it in self.items.items() if it.in_mem and not it.pinned and s != keep]
            v = self._victim(cands, "mem")
            p = None if v is None else self.position(v)
            if v is None or (not_sooner_than is not None and p is not None and p <= not_sooner_than):
                ok = False
            else:
                self._evict_from_memory(v)
        self._keep = None
        return ok

    def _bring_in(self, session, kind):
        i = self.items[session]
        i.in_mem, i.mem_seq = True, self._next_seq()
        self.actions.append((kind, session))
        self.stats["fetched" if kind == FETCH else "loaded"] += 1
        self.stats["bytes_from_disk"] += i.size

    def _expire(self, now):
        if self.ttl <= 0:
            return
        for s in sorted(self.items):
            i = self.items[s]
            if not i.pinned and now - i.last_access > self.ttl:
                i.in_mem = i.on_disk = False
                del self.items[s]
                self.actions.append((EXPIRE, s))
                self.stats["expired"] += 1

    # ---- the calls of the job scheduler ---------------------------------------------------------------
    def set_queue(self, sessions):
        """the waiting jobs' sessions, the next job to run first (the running job is not in it)"""
        self.queue = list(sessions)

    def prefetch(self, now):
        """Section 3.3.1: bring the caches of the first L_pw waiting jobs from disk into memory"""
        self._expire(now)
        if not self.prefetch_on:
            return
        for p, s in enumerate(self.queue[:self.prefetch_window()]):
            i = self.items.get(s)
            if i is None or i.in_mem or not i.on_disk or self.position(s) != p:
                continue
            if i.size > self.mem_capacity:
                continue
            # the buffer is there to be fetched into; it is refilled afterwards
            if not self._make_room(i.size, not_sooner_than=p, keep=s):
                break
            self._bring_in(s, FETCH)
            self._make_room(self.mem_buffer, not_sooner_than=p, keep=s)

    def lookup(self, session, now):
        """a job starts: where is its session's cache?  A disk hit is loaded into memory on the spot."""
        self._expire(now)
        self.stats["lookups"] += 1
        i = self.items.get(session)
        if i is None:
            self.stats["miss"] += 1
            return MISS
        if i.in_mem:
            res = HIT_MEM
            self.stats["hit_mem"] += 1
        else:
            res = HIT_DISK
            self.stats["hit_disk"] += 1
            if i.size <= self.mem_capacity and self._make_room(i.size, keep=session):
                self._bring_in(session, LOAD)
        i.pinned = True
        i.last_access = now
        return res

    def save(self, session, size, now):
        """a job ended: its session's cache, now `size` units, is written back to host memory"""
        assert 0 < size <= self.mem_capacity
        self._expire(now)
        i = self.items.get(session)
        if i is None:
            i = self.items[session] = Item(size, now, self._next_seq())
        i.size = size
        i.pinned = False
        i.last_access = now
        i.on_disk = False                                # whatever the disks hold of it is stale now
        if not i.in_mem:
            i.in_mem, i.mem_seq = True, self._next_seq()
        # first make it fit at all (not at its own expense unless everything else is pinned), then refill the buffer
        i.pinned = True
        ok = self._make_room(0)
        i.pinned = False
        if not ok:
            self._evict_from_memory(session)
        self._make_room(self.mem_buffer)

    def release(self, session, now):
        """a job ended without saving (cancelled, failed): its session is no longer held in memory by a running
        job; the cache stays where it is and the free buffer is restored, now that the item may be moved"""
        self._expire(now)
        i = self.items.get(session)
        if i is None:
            return
        i.pinned = False
        self._make_room(self.mem_buffer)

    def take_actions(self):
        a, self.actions = self.actions, []
        return a
