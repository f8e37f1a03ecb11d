/*
 * ca_store.h - C ABI of the hierarchical KV-cache placement manager (Section 3.3 of
 * arXiv 2403.19708): which conversation sessions' caches are in host memory, which on
 * disk, what is fetched ahead of the job queue and what is evicted.
 *
 * Host-only bookkeeping, no GPU and no I/O: the manager DECIDES; the caller moves the
 * bytes.  Every movement it decides is appended to an action log the caller drains with
 * ca_store_take_actions() and carries out (disk reads and writes, frees).  The KV tier the
 * GPU path of ca.h loads from and saves to is the "host memory" of this manager.
 *
 * One item = all caches of one conversation session, the unit of fetching and eviction
 * (Section 3.3.2).  Sizes and capacities are in one unit of the caller's choice (bytes,
 * tokens, slots).  Sessions are identified by int64 ids.  Times are seconds on any
 * monotonic clock of the caller.
 *
 * The job scheduler's side of the contract:
 *   ca_store_set_queue   whenever the queue of waiting jobs changes (head first, the
 *                        running jobs not included);
 *   ca_store_prefetch    whenever there is time to look ahead (after each queue change);
 *   ca_store_lookup      when a job starts; pins the session in memory;
 *   ca_store_save        when a job ends and its cache has been written back; unpins.
 *   ca_store_release     when a job ends without saving; unpins.
 *
 * Readings of points the section leaves open (they are the manager's behaviour):
 *   - S_kv is the mean size of the items stored at that moment; window lengths are
 *     floor(capacity * items / total size), 0 for an empty store.
 *   - C_mem of both window formulas is mem_capacity - mem_buffer.
 *   - Fetching copies: the disk copy stays valid until the session is saved again; an item
 *     leaving memory with a valid disk copy is released without a write.
 *   - Scheduler-aware order of victims, in memory and on disk: sessions without a job in
 *     the queue first (least recently used first), then the session whose next job is
 *     furthest from the head.  An item with a job inside the look-ahead eviction window
 *     therefore leaves the system only when nothing else is left (counted in
 *     forced_window_drops).  Ties go to the smaller session id.
 *   - When an item leaves memory and the disks are full, it competes with the disk items
 *     under the same order and is itself dropped if it ranks last (scheduler-aware only;
 *     the other two policies always make room on disk).
 *   - A fetch never evicts an item whose job comes sooner than the job fetched for;
 *     prefetching stops at the first job it cannot make room for.
 *
 * Not thread-safe; calls on one store must not overlap.  Nothing throws or aborts.
 */
#ifndef CA_STORE_H_
#define CA_STORE_H_

#include <stdint.h>

#include "ca.h" /* ca_status */

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ca_store ca_store;

enum { CA_STORE_SCHEDULER_AWARE = 0, CA_STORE_LRU = 1, CA_STORE_FIFO = 2 }; /* eviction policy */
enum { CA_STORE_MISS = 0, CA_STORE_HIT_MEM = 1, CA_STORE_HIT_DISK = 2 };    /* lookup result  */
enum { CA_STORE_IN_MEM = 1, CA_STORE_ON_DISK = 2 };                         /* tier bits      */

/* kinds of ca_store_action */
enum {
    CA_STORE_FETCH = 1,     /* disk -> memory ahead of the job (Section 3.3.1); disk copy stays   */
    CA_STORE_LOAD = 2,      /* disk -> memory on demand: the job started with its cache on disk    */
    CA_STORE_EVICT = 3,     /* memory -> disk, written (Section 3.3.2)                             */
    CA_STORE_RELEASE = 4,   /* memory copy freed, the disk copy was still valid: no write          */
    CA_STORE_DROP_DISK = 5, /* disk copy freed, the item stays in memory                           */
    CA_STORE_DROP = 6,      /* the item leaves the system                                          */
    CA_STORE_EXPIRE = 7     /* the item leaves the system: not touched for longer than ttl         */
};

typedef struct {
    int64_t mem_capacity;  /* host memory for caches, >= 0                                        */
    int64_t disk_capacity; /* >= 0; 0 = no disk tier                                              */
    int64_t mem_buffer;    /* part of mem_capacity kept free so that fetches never wait for an
                              eviction (Section 3.3.1, last paragraph); 0 <= mem_buffer <= mem_capacity */
    int32_t policy;        /* CA_STORE_SCHEDULER_AWARE / _LRU / _FIFO                              */
    int32_t prefetch;      /* 1: ca_store_prefetch fetches; 0: it only expires                     */
    double ttl;            /* time to live since the last access (Section 4.5); <= 0: none         */
} ca_store_config;

typedef struct {
    int32_t kind;
    int32_t reserved;
    int64_t session;
} ca_store_action;

typedef struct {
    int64_t lookups, hit_mem, hit_disk, miss;
    int64_t fetched, loaded, evicted, released, dropped, expired;
    int64_t forced_window_drops; /* items dropped although a job of theirs was inside the eviction window */
    int64_t bytes_to_disk, bytes_from_disk; /* in the caller's size unit */
} ca_store_stats;

/* Section 3.3.  Creates an empty store.  CA_ERR_INVALID_ARG for a null pointer, a negative
 * capacity, a buffer larger than the memory, an unknown policy. */
ca_status ca_store_create(const ca_store_config *cfg, ca_store **out);
void ca_store_destroy(ca_store *store);
/* text of the last failure on this store (owned by the store, valid until the next call) */
const char *ca_store_last_error(const ca_store *store);

/* Places an item directly (a state restored at start-up).  tiers: CA_STORE_IN_MEM and/or
 * CA_STORE_ON_DISK.  CA_ERR_INVALID_ARG if the session is already known, size <= 0 or
 * tiers is 0; CA_ERR_OUT_OF_RANGE if a capacity would be exceeded. */
ca_status ca_store_seed(ca_store *store, int64_t session, int64_t size, int32_t tiers, double now);

/* Sections 3.3.1 / 3.3.2: the scheduler's knowledge of the future.  sessions[0..n) are the
 * sessions of the waiting jobs, the next one to run first; copied.  n = 0 empties it. */
ca_status ca_store_set_queue(ca_store *store, const int64_t *sessions, int32_t n);

/* Section 3.3.1: for the first L_pw = C_mem / S_kv waiting jobs, fetches the caches found
 * on disk into memory, evicting (Section 3.3.2) to keep mem_buffer free.  Also expires. */
ca_status ca_store_prefetch(ca_store *store, double now);

/* A job starts.  *where = CA_STORE_MISS / _HIT_MEM / _HIT_DISK; a disk hit is loaded into
 * memory on the spot (evicting if needed).  The session stays pinned until ca_store_save
 * or ca_store_release. */
ca_status ca_store_lookup(ca_store *store, int64_t session, double now, int32_t *where);

/* A job ended: the session's cache, now `size` units, is in host memory (Section 3.2.2
 * wrote it there).  Any disk copy becomes stale and is forgotten.  Evicts to restore
 * mem_buffer.  CA_ERR_OUT_OF_RANGE if size > mem_capacity, CA_ERR_INVALID_ARG if size <= 0. */
ca_status ca_store_save(ca_store *store, int64_t session, int64_t size, double now);

/* A job ended WITHOUT saving (cancelled, failed, read-only): the session is no longer pinned;
 * its cache stays where it is and mem_buffer is restored.  Unknown sessions are ignored. */
ca_status ca_store_release(ca_store *store, int64_t session, double now);

/* *tiers = tier bits of the session (0: unknown to the store). */
ca_status ca_store_where(const ca_store *store, int64_t session, int32_t *tiers);
/* L_pw (Section 3.3.1) and the look-ahead eviction window length (Section 3.3.2), now. */
ca_status ca_store_windows(const ca_store *store, int64_t *prefetch_window, int64_t *eviction_window);
ca_status ca_store_usage(const ca_store *store, int64_t *mem_used, int64_t *disk_used, int64_t *n_items);
ca_status ca_store_stats_read(const ca_store *store, ca_store_stats *out);

/* Copies the pending actions, oldest first, into out[0..capacity) and clears the log.
 * *count = number of pending actions; if it exceeds capacity nothing is copied or cleared
 * and CA_ERR_OUT_OF_RANGE is returned.  out may be NULL when capacity is 0. */
ca_status ca_store_take_actions(ca_store *store, ca_store_action *out, int64_t capacity, int64_t *count);

#ifdef __cplusplus
}
#endif
#endif /* CA_STORE_H_ */
