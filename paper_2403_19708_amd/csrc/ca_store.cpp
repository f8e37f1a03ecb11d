// Hierarchical KV-cache placement manager (Section 3.3): host-side bookkeeping of which sessions'
// caches are in host memory and which on disk, the scheduler-aware fetching of Section 3.3.1 and the
// scheduler-aware eviction of Section 3.3.2, with least-recently-used and first-in-first-out eviction
// as the alternatives the evaluation compares against.  Decides only; the caller moves the bytes.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <new>
#include <unordered_map>
#include <vector>

#include "../../include/ca_store.h"

namespace {

struct Entry {
    int64_t size = 0;
    bool in_mem = false, on_disk = false, pinned = false;
    double last_access = 0.0;
    uint64_t mem_order = 0, disk_order = 0;  // arrival order in the tier
};

// Eviction priority: the smallest key goes first.
struct Key {
    int cls;
    double t;
    int64_t n;
    int64_t id;
    bool operator<(const Key &o) const {
        if (cls != o.cls) return cls < o.cls;
        if (t != o.t) return t < o.t;
        if (n != o.n) return n < o.n;
        return id < o.id;
    }
};

enum class Tier { kMem, kDisk };

}  // namespace

struct ca_store {
    ca_store_config cfg{};
    std::unordered_map<int64_t, Entry> entries;
    std::unordered_map<int64_t, int32_t> first_pos;  // session -> position of its first waiting job
    std::vector<int64_t> queue;
    std::vector<ca_store_action> log;
    ca_store_stats stats{};
    int64_t mem_used = 0, disk_used = 0, total_size = 0;
    uint64_t order = 0;
    int64_t shielded = -1;  // session being brought into memory: neither copy of it is a victim
    bool has_shield = false;
    char err[256] = {0};

    ca_status fail(ca_status st, const char *fmt, ...) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(err, sizeof err, fmt, ap);
        va_end(ap);
        return st;
    }

    int64_t window(int64_t capacity) const {
        // capacity / S_kv with S_kv = total_size / count, in whole numbers
        if (total_size <= 0) return 0;
        return (int64_t)(((__int128)capacity * (int64_t)entries.size()) / total_size);
    }
    int64_t prefetch_window() const { return window(cfg.mem_capacity - cfg.mem_buffer); }
    int64_t eviction_window() const { return window(cfg.mem_capacity - cfg.mem_buffer + cfg.disk_capacity); }

    int32_t pos_of(int64_t id) const {
        auto it = first_pos.find(id);
        return it == first_pos.end() ? -1 : it->second;
    }

    Key key_of(int64_t id, const Entry &e, Tier tier) const {
        switch (cfg.policy) {
            case CA_STORE_LRU: return {0, e.last_access, 0, id};
            case CA_STORE_FIFO: return {0, 0.0, (int64_t)(tier == Tier::kMem ? e.mem_order : e.disk_order), id};
            default: {
                const int32_t p = pos_of(id);
                if (p < 0) return {0, e.last_access, 0, id};  // no waiting job: by recency
                return {1, 0.0, -(int64_t)p, id};             // waiting: the one furthest from the head first
            }
        }
    }

    void record(int32_t kind, int64_t id) { log.push_back({kind, 0, id}); }

    void note_drop(int64_t id) {
        record(CA_STORE_DROP, id);
        stats.dropped++;
        const int32_t p = pos_of(id);
        if (p >= 0 && p < eviction_window()) stats.forced_window_drops++;
    }

    void erase_if_gone(int64_t id) {
        auto it = entries.find(id);
        if (it != entries.end() && !it->second.in_mem && !it->second.on_disk) {
            total_size -= it->second.size;
            entries.erase(it);
        }
    }

    // best victim among the copies one tier holds (pinned and shielded items are never candidates)
    bool pick(Tier tier, int64_t *out) const {
        bool found = false;
        Key best{};
        for (const auto &kv : entries) {
            const Entry &e = kv.second;
            if (has_shield && kv.first == shielded) continue;
            if (tier == Tier::kMem ? (!e.in_mem || e.pinned) : !e.on_disk) continue;
            const Key k = key_of(kv.first, e, tier);
            if (!found || k < best) { best = k; *out = kv.first; found = true; }
        }
        return found;
    }

    void free_disk_copy(int64_t id) {
        Entry &e = entries.at(id);
        e.on_disk = false;
        disk_used -= e.size;
        if (e.in_mem) {
            record(CA_STORE_DROP_DISK, id);
        } else {
            note_drop(id);
            erase_if_gone(id);
        }
    }

    // Section 3.3.2: one item leaves memory for the disks (or the system, if the disks cannot take it)
    void leave_memory(int64_t id) {
        Entry &e = entries.at(id);
        if (e.on_disk) {
            e.in_mem = false;
            mem_used -= e.size;
            record(CA_STORE_RELEASE, id);
            stats.released++;
            return;
        }
        const int64_t size = e.size;
        while (size > cfg.disk_capacity - disk_used) {
            int64_t victim = id;
            bool any = false;
            if (size <= cfg.disk_capacity) {
                // the incoming item competes only under the scheduler-aware order
                int64_t v;
                if (pick(Tier::kDisk, &v)) {
                    any = true;
                    victim = v;
                    if (cfg.policy == CA_STORE_SCHEDULER_AWARE && key_of(id, entries.at(id), Tier::kDisk) < key_of(v, entries.at(v), Tier::kDisk))
                        victim = id;
                }
            }
            if (!any || victim == id) {
                Entry &self = entries.at(id);
                self.in_mem = false;
                mem_used -= self.size;
                note_drop(id);
                erase_if_gone(id);
                return;
            }
            free_disk_copy(victim);
        }
        Entry &self = entries.at(id);
        self.in_mem = false;
        self.on_disk = true;
        self.disk_order = ++order;
        mem_used -= size;
        disk_used += size;
        record(CA_STORE_EVICT, id);
        stats.evicted++;
        stats.bytes_to_disk += size;
    }

    // Evicts until `need_free` units of memory are free.  limit_pos >= 0: never at the expense of an item
    // whose job waits at or before that queue position.  shield: the session being brought in.
    bool make_room(int64_t need_free, int32_t limit_pos, bool shield, int64_t shield_id) {
        has_shield = shield;
        shielded = shield_id;
        bool ok = true;
        while (ok && cfg.mem_capacity - mem_used < need_free) {
            int64_t v;
            if (!pick(Tier::kMem, &v)) {
                ok = false;
            } else {
                const int32_t p = pos_of(v);
                if (limit_pos >= 0 && p >= 0 && p <= limit_pos) ok = false;
                else leave_memory(v);
            }
        }
        has_shield = false;
        return ok;
    }

    void bring_in(int64_t id, int32_t kind) {
        Entry &e = entries.at(id);
        e.in_mem = true;
        e.mem_order = ++order;
        mem_used += e.size;
        record(kind, id);
        (kind == CA_STORE_FETCH ? stats.fetched : stats.loaded)++;
        stats.bytes_from_disk += e.size;
    }

    void expire(double now) {
        if (!(cfg.ttl > 0.0)) return;
        std::vector<int64_t> gone;
        for (const auto &kv : entries)
            if (!kv.second.pinned && now - kv.second.last_access > cfg.ttl) gone.push_back(kv.first);
        std::sort(gone.begin(), gone.end());
        for (int64_t id : gone) {
            Entry &e = entries.at(id);
            if (e.in_mem) mem_used -= e.size;
            if (e.on_disk) disk_used -= e.size;
            total_size -= e.size;
            entries.erase(id);
            record(CA_STORE_EXPIRE, id);
            stats.expired++;
        }
    }
};

extern "C" {

ca_status ca_store_create(const ca_store_config *cfg, ca_store **out) {
    if (!cfg || !out) return CA_ERR_INVALID_ARG;
    *out = nullptr;
    if (cfg->mem_capacity < 0 || cfg->disk_capacity < 0 || cfg->mem_buffer < 0 || cfg->mem_buffer > cfg->mem_capacity)
        return CA_ERR_INVALID_ARG;
    if (cfg->policy != CA_STORE_SCHEDULER_AWARE && cfg->policy != CA_STORE_LRU && cfg->policy != CA_STORE_FIFO)
        return CA_ERR_INVALID_ARG;
    if (cfg->prefetch != 0 && cfg->prefetch != 1) return CA_ERR_INVALID_ARG;
    ca_store *s = new (std::nothrow) ca_store();
    if (!s) return CA_ERR_NOMEM;
    s->cfg = *cfg;
    *out = s;
    return CA_OK;
}

void ca_store_destroy(ca_store *store) { delete store; }

const char *ca_store_last_error(const ca_store *store) { return store ? store->err : "null store"; }

ca_status ca_store_seed(ca_store *s, int64_t session, int64_t size, int32_t tiers, double now) {
    if (!s) return CA_ERR_INVALID_ARG;
    if (size <= 0 || (tiers & ~3) || !(tiers & 3)) return s->fail(CA_ERR_INVALID_ARG, "ca_store_seed: size %lld, tiers %d", (long long)size, tiers);
    if (s->entries.count(session)) return s->fail(CA_ERR_INVALID_ARG, "ca_store_seed: session %lld is already stored", (long long)session);
    const bool m = tiers & CA_STORE_IN_MEM, d = tiers & CA_STORE_ON_DISK;
    if ((m && s->mem_used + size > s->cfg.mem_capacity) || (d && s->disk_used + size > s->cfg.disk_capacity))
        return s->fail(CA_ERR_OUT_OF_RANGE, "ca_store_seed: session %lld does not fit", (long long)session);
    Entry e;
    e.size = size;
    e.in_mem = m;
    e.on_disk = d;
    e.last_access = now;
    e.mem_order = e.disk_order = ++s->order;
    s->entries.emplace(session, e);
    s->total_size += size;
    if (m) s->mem_used += size;
    if (d) s->disk_used += size;
    return CA_OK;
}

ca_status ca_store_set_queue(ca_store *s, const int64_t *sessions, int32_t n) {
    if (!s) return CA_ERR_INVALID_ARG;
    if (n < 0 || (n > 0 && !sessions)) return s->fail(CA_ERR_INVALID_ARG, "ca_store_set_queue: n = %d", n);
    s->queue.assign(sessions, sessions + n);
    s->first_pos.clear();
    s->first_pos.reserve((size_t)n);
    for (int32_t i = 0; i < n; ++i) s->first_pos.emplace(sessions[i], i);  // emplace keeps the first occurrence
    return CA_OK;
}

ca_status ca_store_prefetch(ca_store *s, double now) {
    if (!s) return CA_ERR_INVALID_ARG;
    s->expire(now);
    if (!s->cfg.prefetch) return CA_OK;
    const int64_t reach = std::min<int64_t>(s->prefetch_window(), (int64_t)s->queue.size());
    for (int64_t p = 0; p < reach; ++p) {
        const int64_t id = s->queue[(size_t)p];
        auto it = s->entries.find(id);
        if (it == s->entries.end() || it->second.in_mem || !it->second.on_disk) continue;
        if (s->pos_of(id) != (int32_t)p) continue;           // a later job of a session already looked at
        const int64_t size = it->second.size;
        if (size > s->cfg.mem_capacity) continue;
        // the free buffer is what the fetch lands in; it is refilled right after
        if (!s->make_room(size, (int32_t)p, true, id)) break;
        s->bring_in(id, CA_STORE_FETCH);
        (void)s->make_room(s->cfg.mem_buffer, (int32_t)p, true, id);
    }
    return CA_OK;
}

ca_status ca_store_lookup(ca_store *s, int64_t session, double now, int32_t *where) {
    if (!s) return CA_ERR_INVALID_ARG;
    if (!where) return s->fail(CA_ERR_INVALID_ARG, "ca_store_lookup: where is NULL");
    s->expire(now);
    s->stats.lookups++;
    auto it = s->entries.find(session);
    if (it == s->entries.end()) {
        s->stats.miss++;
        *where = CA_STORE_MISS;
        return CA_OK;
    }
    if (it->second.in_mem) {
        s->stats.hit_mem++;
        *where = CA_STORE_HIT_MEM;
    } else {
        s->stats.hit_disk++;
        *where = CA_STORE_HIT_DISK;
        const int64_t size = it->second.size;
        if (size <= s->cfg.mem_capacity && s->make_room(size, -1, true, session)) s->bring_in(session, CA_STORE_LOAD);
    }
    Entry &e = s->entries.at(session);
    e.pinned = true;
    e.last_access = now;
    return CA_OK;
}

ca_status ca_store_save(ca_store *s, int64_t session, int64_t size, double now) {
    if (!s) return CA_ERR_INVALID_ARG;
    if (size <= 0) return s->fail(CA_ERR_INVALID_ARG, "ca_store_save: size %lld", (long long)size);
    if (size > s->cfg.mem_capacity)
        return s->fail(CA_ERR_OUT_OF_RANGE, "ca_store_save: size %lld exceeds the memory capacity %lld", (long long)size, (long long)s->cfg.mem_capacity);
    s->expire(now);
    Entry &e = s->entries[session];  // created empty if new
    s->total_size += size - e.size;
    if (e.in_mem) s->mem_used += size - e.size;
    if (e.on_disk) {                 // stale from now on
        s->disk_used -= e.size;
        e.on_disk = false;
    }
    e.size = size;
    e.last_access = now;
    if (!e.in_mem) {
        e.in_mem = true;
        e.mem_order = ++s->order;
        s->mem_used += size;
    }
    // it has to fit first, at the others' expense; only then is the buffer refilled, where it competes too
    e.pinned = true;
    const bool fits = s->make_room(0, -1, false, 0);
    s->entries.at(session).pinned = false;
    if (!fits) s->leave_memory(session);
    (void)s->make_room(s->cfg.mem_buffer, -1, false, 0);
    return CA_OK;
}

ca_status ca_store_release(ca_store *s, int64_t session, double now) {
    if (!s) return CA_ERR_INVALID_ARG;
    s->expire(now);
    auto it = s->entries.find(session);
    if (it == s->entries.end()) return CA_OK;
    it->second.pinned = false;
    (void)s->make_room(s->cfg.mem_buffer, -1, false, 0);
    return CA_OK;
}

ca_status ca_store_where(const ca_store *s, int64_t session, int32_t *tiers) {
    if (!s || !tiers) return CA_ERR_INVALID_ARG;
    auto it = s->entries.find(session);
    *tiers = it == s->entries.end() ? 0 : (it->second.in_mem ? CA_STORE_IN_MEM : 0) | (it->second.on_disk ? CA_STORE_ON_DISK : 0);
    return CA_OK;
}

ca_status ca_store_windows(const ca_store *s, int64_t *prefetch_window, int64_t *eviction_window) {
    if (!s || !prefetch_window || !eviction_window) return CA_ERR_INVALID_ARG;
    *prefetch_window = s->prefetch_window();
    *eviction_window = s->eviction_window();
    return CA_OK;
}

ca_status ca_store_usage(const ca_store *s, int64_t *mem_used, int64_t *disk_used, int64_t *n_items) {
    if (!s || !mem_used || !disk_used || !n_items) return CA_ERR_INVALID_ARG;
    *mem_used = s->mem_used;
    *disk_used = s->disk_used;
    *n_items = (int64_t)s->entries.size();
    return CA_OK;
}

ca_status ca_store_stats_read(const ca_store *s, ca_store_stats *out) {
    if (!s || !out) return CA_ERR_INVALID_ARG;
    *out = s->stats;
    return CA_OK;
}

ca_status ca_store_take_actions(ca_store *s, ca_store_action *out, int64_t capacity, int64_t *count) {
    if (!s) return CA_ERR_INVALID_ARG;
    if (!count || capacity < 0 || (capacity > 0 && !out)) return s->fail(CA_ERR_INVALID_ARG, "ca_store_take_actions: bad arguments");
    *count = (int64_t)s->log.size();
    if (*count > capacity) return s->fail(CA_ERR_OUT_OF_RANGE, "ca_store_take_actions: %lld actions pending, capacity %lld", (long long)*count, (long long)capacity);
    std::copy(s->log.begin(), s->log.end(), out);
    s->log.clear();
    return CA_OK;
}

}  // extern "C"
