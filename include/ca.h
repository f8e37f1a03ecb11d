/*
 * ca.h - C ABI of the CachedAttention new-turn prefill path for AMD MI355X (gfx950).
 *
 * The library implements, as hand-written HIP kernels on ONE GPU, the part of
 * CachedAttention (arXiv 2403.19708) that runs for every new conversation turn:
 *
 *   save   (Section 3.2.2) keys/values leave HBM layer by layer on a write stream; keys
 *                          are stored WITHOUT positional encoding (Section 3.4).
 *   load   (Section 3.2.1) the saved history of layer l is brought back into the paged
 *                          HBM pool on a read stream while earlier layers compute.
 *   rebase (Section 3.4)   after context-window truncation the kept tokens are numbered
 *                          again from 0; the rotary encoding is embedded at these new
 *                          positions when the cache is used.
 *   attend (Sections 2.1, 3.1) only the new tokens are prefilled: their queries attend
 *                          to [kept history | new tokens] with a causal mask.
 *
 * Conventions
 *   - Plain C types only.  "device" pointers are HIP device memory, "host" pointers are
 *     ordinary host memory unless "pinned" is stated (then hipHostMalloc'd / torch
 *     pin_memory).  Streams are hipStream_t passed as void*; NULL is the default stream.
 *   - The caller owns every tensor (pools, Q, output, host tier).  The library owns its
 *     context: three internal streams (copy-in, unpack, save), events, a ring of staging
 *     slots in HBM, a rotary table and small per-batch metadata.  It never frees or
 *     reallocates caller memory.
 *   - Every call validates its arguments on the host BEFORE anything is launched and
 *     returns a ca_status; nothing throws or aborts.  ca_last_error() gives the text of
 *     the last failure on that context.  A context is not thread-safe.
 *   - All entry points except ca_create / ca_destroy / ca_sync / ca_rebase_read are
 *     asynchronous with respect to the host.
 *
 * Layouts (element type bf16 = 2 bytes unless stated)
 *   paged pool   k_pool, v_pool : [num_pages][n_kv_heads][page_size][head_dim], one pair
 *                per layer; keys in the pool carry NO positional encoding.
 *   contiguous   per conversation and layer: [tokens][n_kv_heads][head_dim] (what the
 *                host tier stores; token 0 is the oldest saved token).
 *   q, out       [sum new_len][n_q_heads][head_dim], conversations concatenated in batch
 *                order; q carries NO positional encoding.
 *   block_table  [n_seqs][max_pages] int32 physical page ids; context token t of
 *                conversation c lives in page block_table[c][t / page_size], slot
 *                t % page_size.  The context of c is [kept history | new tokens].
 *   Query head h reads KV head h / (n_q_heads / n_kv_heads).
 */
#ifndef CA_H_
#define CA_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ca_ctx ca_ctx;

typedef enum {
    CA_OK = 0,
    CA_ERR_INVALID_ARG = 1,  /* null pointer, negative size, inconsistent lengths            */
    CA_ERR_OUT_OF_RANGE = 2, /* layer, page id, token range or batch size beyond a limit      */
    CA_ERR_UNSUPPORTED = 3,  /* head_dim / page_size / style the kernels are not built for    */
    CA_ERR_NOMEM = 4,        /* context allocation failed                                     */
    CA_ERR_NOT_READY = 5,    /* call order: no rebase yet, layer not loaded, loaded twice     */
    CA_ERR_HIP = 6           /* a HIP runtime call failed; text in ca_last_error()            */
} ca_status;

typedef struct {
    int32_t n_layers;
    int32_t n_q_heads;
    int32_t n_kv_heads;      /* divides n_q_heads                                             */
    int32_t head_dim;        /* 64 or 128                                                     */
    int32_t page_size;       /* tokens per page; 16                                           */
    int32_t max_positions;   /* context window W: largest context (kept history + new) + 0    */
    float   rope_base;       /* 10000                                                         */
    int32_t rope_style;      /* 0: pairs (i, i + head_dim/2); 1: pairs (2i, 2i+1)             */
    int32_t pipeline_depth;  /* staging slots for loads (read buffer) and for saves, >= 1     */
    int32_t max_seqs;        /* largest batch                                                 */
    int64_t max_batch_kv_tokens; /* largest sum over the batch of context tokens; sizes one   */
                                 /* staging slot and the metadata                             */
    int64_t max_batch_q_tokens;  /* largest sum over the batch of new tokens                  */
    int32_t load_mode;       /* 0: choose per source pointer; 1: copy into a staging slot,    */
                             /* then unpack; 2: the unpack kernel reads the source in place   */
                             /* (source must be device-accessible)                            */
    int32_t save_mode;       /* for ca_kv_save_layer / ca_kv_append_save_layer.  Device memory is  */
                             /* written in place by the pack kernel unless 1.  Pinned host memory: */
                             /* 1 pack into a staging slot, then one copy per conversation on a    */
                             /* copy engine (about 8 GB/s for turns of a few hundred tokens, and   */
                             /* disturbs no kernel); 2 the pack kernel stores over the host link   */
                             /* from the internal save stream (about 40 GB/s, but kernels running  */
                             /* beside it are held up for about as long as it runs; with 2         */
                             /* ca_kv_append_save_layer stores from the one kernel on the caller's */
                             /* stream); 0 chooses per call: staged while the tokens to save are   */
                             /* fewer than a fifth of the kept history loaded per layer (the       */
                             /* copies then hide under the load), else in place                    */
    int32_t attn_variant;    /* 0: choose (the streaming kernel for a batch of decode steps, else the    */
                             /* matrix-core kernel); 1: scalar fp32 kernel (slow, for checking); 2: the  */
                             /* matrix-core kernel, K/V loaded straight into LDS, whatever the batch;    */
                             /* 4: as 0, but a batch in which some (conversation, kv head) has more than */
                             /* 2 stacked query rows (not a decode step) is refused by                   */
                             /* ca_cached_prefill_attn with CA_ERR_UNSUPPORTED.  (3 named a second       */
                             /* matrix-core kernel that was removed; it is refused.)                     */
    int32_t attn_tile_rows;  /* stacked query rows per workgroup of the MFMA kernel: 128, 256,  */
                             /* or 0 = choose per batch                                        */
    int32_t attn_split;      /* 0: when a batch has too few row tiles to keep all compute units */
                             /* busy, the LDS-direct kernel splits the keys of long tiles over  */
                             /* several workgroups and merges their shares; 1: never split      */
    int32_t attn_prerotate;  /* the LDS-direct kernel applies the rotary encoding to a key in    */
                             /* every row tile that reads it; when many row tiles share the keys */
                             /* of a (conversation, kv head) (long new turns, grouped heads) it  */
                             /* is cheaper to rotate the batch's keys once per layer into a      */
                             /* scratch copy first.  0: decide per batch (three or more 256-row  */
                             /* tiles per (conversation, kv head) on average); 1: never;         */
                             /* 2: always (256-row tiles are then used whatever the batch)       */
    int32_t attn_schedule;   /* 0: the LDS-direct kernel, all wavefronts of a workgroup in lock step.      */
                             /* 1: when the keys are rotated once per layer (attn_prerotate), head_dim is  */
                             /* 128 and the tiles have 256 rows, the values are transposed into a scratch  */
                             /* copy in the same pass and a kernel runs that pipelines, inside every       */
                             /* wavefront, the matrix instructions of one key tile with the softmax of the */
                             /* previous one (any window; measured as fast as 0, plus the longer pre-pass)  */
    int32_t require_load;    /* 1: attention on a layer with kept history that was not loaded */
                             /* under the current plan fails with CA_ERR_NOT_READY            */
    int32_t device;          /* HIP device ordinal                                            */
} ca_config;

/* One batch of conversations about to run a new turn.  All pointers are HOST memory and are
 * read during ca_rope_rebase only.  keep_start[c] in [0, hist_len[c]] is the first saved token
 * that survives truncation; n_keep = hist_len - keep_start; context = n_keep + new_len.
 * A token discarding list (Section 3.4, last paragraph) is given as its complement: the kept
 * saved tokens of conversation c are the union of keep_range_count[c] ranges [begin, end) taken
 * in order from keep_ranges; inside a conversation the ranges are non-empty, increasing and
 * disjoint, inside [0, hist_len[c]].  n_keep is then the sum of their lengths, the kept tokens
 * are renumbered densely from 0 in that order, and keep_start is not read.                     */
typedef struct {
    int32_t n_seqs;
    const int32_t *hist_len;    /* [n_seqs] tokens saved in the host tier                     */
    const int32_t *keep_start;  /* [n_seqs]; may be NULL when keep_ranges is given            */
    const int32_t *new_len;     /* [n_seqs] >= 1                                              */
    const int32_t *block_table; /* [n_seqs][max_pages]; the first ceil(context/page_size)     */
                                /* entries of a row must be distinct valid pages              */
    int32_t max_pages;
    int32_t num_pages;          /* pages in every pool later passed with this batch           */
    const int32_t *keep_ranges;       /* NULL, or [sum keep_range_count][2] (begin, end)      */
    const int32_t *keep_range_count;  /* NULL iff keep_ranges is NULL; [n_seqs], each >= 0    */
} ca_batch;

/* ---- context ------------------------------------------------------------------------ */

/* Fills *cfg with defaults (page 16, base 10000, half-split pairs, depth 2, attention kernel
 * chosen by the window, key splitting on).                                                  */
void ca_config_default(ca_config *cfg);

/* Host-only checks of a configuration / a batch against a configuration.  Used by every
 * entry point; exported so that callers (and CPU-only tests) can check without a GPU.
 * err, if not NULL, receives a message of at most err_len bytes.                           */
ca_status ca_config_validate(const ca_config *cfg, char *err, int32_t err_len);
ca_status ca_batch_validate(const ca_config *cfg, const ca_batch *batch, char *err, int32_t err_len);

/* Allocates the context on cfg->device: streams, events, staging ring
 * (2 * pipeline_depth slots of 2 * max_batch_kv_tokens * n_kv_heads * head_dim * 2 bytes),
 * rotary table (max_positions * head_dim/2 cos/sin pairs, fp32, computed in fp64), metadata. */
ca_status ca_create(const ca_config *cfg, ca_ctx **out);
void ca_destroy(ca_ctx *ctx);
const char *ca_last_error(const ca_ctx *ctx);
const char *ca_status_string(ca_status s);

/* ---- Section 3.4 / 4.1: truncation planner (host only, no context needed) ----------- */
/* keep_start_out[c] = 0 unless hist_len[c] + new_len[c] > window.  On overflow the most recent
 * tokens survive:  policy 0 keeps floor(window*(1-ratio)) tokens of [history|new] (the new turn
 * is never dropped); policy 1 drops floor(window*ratio) oldest tokens, repeatedly while the
 * context still overflows; policy 2 drops floor(ratio*context) oldest tokens, repeatedly.
 * 0 < ratio < 1.  Arrays are host memory of n entries.                                       */
ca_status ca_truncate_plan(const int32_t *hist_len, const int32_t *new_len, int32_t window,
                           double ratio, int32_t policy, int32_t n, int32_t *keep_start_out);

/* The same overflow rule as policy 0, with a discarding list that spares the first n_sink saved
 * tokens (Section 3.4, last paragraph: keeping chosen tokens, for instance the first ones of a
 * text, instead of a plain suffix): without overflow
 * conversation c keeps one range [0, hist_len); on overflow it keeps floor(window*(1-ratio)) -
 * new_len history tokens (0 if negative): the first min(n_sink, that many) and the most recent
 * rest.  ranges_out: [n][2][2] (two (begin, end) slots per conversation, unused ones 0, 0);
 * count_out[c] in {0, 1, 2}; adjacent pieces are merged into one range.  To pass the result as
 * ca_batch.keep_ranges, compact the used slots in order.                                      */
ca_status ca_truncate_plan_sinks(const int32_t *hist_len, const int32_t *new_len, int32_t window,
                                 double ratio, int32_t n_sink, int32_t n, int32_t *ranges_out,
                                 int32_t *count_out);

/* Section 3.4, last paragraph: drops the discarded tokens from the saved cache itself.  For every
 * conversation the rows of its kept tokens -- the ranges of keep_ranges / keep_range_count exactly
 * as in ca_batch, or [keep_start[c], hist_len[c]) when keep_ranges is NULL -- are moved to the
 * front of tier_k[c] and tier_v[c] in order, and hist_len_out[c] receives how many rows are left
 * (pass it as hist_len, with keep_start 0, from then on).  One layer's buffers per call.
 * tier_k / tier_v: HOST memory (pinned or not), [hist_len[c]] rows of row_bytes =
 * n_kv_heads * head_dim * 2 bytes; the move is done by the calling thread with memmove, so no
 * load or save of these buffers may be in flight (ca_sync first).  Arguments are checked before
 * anything moves: CA_ERR_OUT_OF_RANGE for ranges that are empty, not increasing, overlapping or
 * outside [0, hist_len].  Needs no context and no GPU.                                          */
ca_status ca_tier_compact(int32_t n_seqs, const int32_t *hist_len, const int32_t *keep_start,
                          const int32_t *keep_ranges, const int32_t *keep_range_count,
                          int64_t row_bytes, void *const *tier_k, void *const *tier_v,
                          int32_t *hist_len_out);

/* ---- Section 3.4: position rebasing --------------------------------------------------- */
/* Makes `batch` the context's current plan: numbers the kept tokens of every conversation
 * from 0 (keys 0..context-1, new token j at n_keep + j), and builds on the device the
 * metadata the other calls use (prefix sums, per-token positions and page slots, the
 * attention work list).  Host arrays of `batch` may be reused when the call returns.
 * Ordering: work queued earlier on `stream` and on the internal streams completes before
 * the metadata changes; later calls on this context see the new plan.                       */
ca_status ca_rope_rebase(ca_ctx *ctx, const ca_batch *batch, void *stream);

/* Copies a piece of the current plan's device metadata to host (synchronises; for tests and
 * debugging).  which: 0 n_keep[n_seqs], 1 cu_q[n_seqs+1], 2 cu_k[n_seqs+1], 3 q_pos[sum new],
 * 4 q_seq[sum new], 5 slot_map[sum context] (page*page_size + slot of every context token),
 * 6 attention work list (8 int32 per item: seq, kv_head, first_row, n_rows, key_begin, key_end,
 *   part, 0; seq -1 = padding; part -1 = the item covers all keys its rows see, else the item is
 *   one share of a row tile whose keys [key_begin, key_end) were split over workgroups).
 * capacity is in int32 elements; *count receives the number written.                         */
ca_status ca_rebase_read(ca_ctx *ctx, int32_t which, int32_t *out, int64_t capacity, int64_t *count);

/* ---- Section 3.2.1: layer-wise loading -------------------------------------------------- */
/* Brings the kept history of `layer` into the pools: for every conversation c the tokens
 * [keep_start[c], hist_len[c]) of src_k[c] / src_v[c] (contiguous layout, pointer to saved
 * token 0 of this layer; host array of n_seqs pointers) -- or, with a discarding list, the
 * tokens of its kept ranges in order -- become context tokens [0, n_keep[c]).
 * Truncation and discarding are just source offsets.  Runs on the internal copy-in and unpack streams and
 * marks the layer ready; ca_cached_prefill_attn(layer) waits for that mark on its own stream.
 * Sources: pinned host memory (staged hipMemcpyAsync into a ring slot + unpack kernel -- the K
 * half is copied on the copy-in stream and the V half on the unpack stream, two copy queues
 * keeping the host link busier than one -- or read in place by the unpack kernel, see load_mode)
 * or device memory (read in place).  A layer can be loaded once per plan (CA_ERR_NOT_READY
 * otherwise).                                                                                  */
ca_status ca_kv_load_layer(ca_ctx *ctx, int32_t layer, const void *const *src_k,
                           const void *const *src_v, void *k_pool, void *v_pool);

/* Writes the new turn's keys/values (device, [sum new_len][n_kv_heads][head_dim], no positional
 * encoding) behind the kept history, context tokens [n_keep[c], n_keep[c]+new_len[c]), on
 * `stream`.  This is the hand-over point from the K/V projections of a model.                 */
ca_status ca_kv_append_layer(ca_ctx *ctx, int32_t layer, const void *new_k, const void *new_v,
                             void *k_pool, void *v_pool, void *stream);

/* ---- Sections 2.1, 3.1, 3.4: prefill of the new tokens over the reused cache ------------ */
/* out[j, h, :] = sum_t softmax_t( RoPE(q[j,h], n_keep+j) . RoPE(k[t, h/G], t) * softmax_scale ) v[t, h/G]
 * over context tokens t <= n_keep + j of the same conversation.  The rotary encoding is applied
 * to keys as they are read from the pool; the pool is not modified.  bf16 in, fp32 accumulate,
 * bf16 out.  q, out: device.  Waits (on `stream`) for the load of `layer` if one was issued.   */
ca_status ca_cached_prefill_attn(ca_ctx *ctx, int32_t layer, const void *q, const void *k_pool,
                                 const void *v_pool, void *out, float softmax_scale, void *stream);

/* The same call for callers that cannot allocate device memory or tolerate a library that does:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Identical
 * arguments, kernels and results; the one scratch buffer the attention kernels use beyond inputs
 * and outputs -- the partial results (fp32 sums, maxima, denominators) of row tiles whose keys the
 * plan split over several workgroups -- is taken from a fixed 32 MiB array inside the library's
 * code object (one copy per GPU, held until the process ends) instead of the context's buffer.
 * The call allocates nothing and records no timing intervals.  A plan whose shares need more than
 * 32 MiB (n_shares * tile_rows * (head_dim + 2) * 4 bytes) is refused with CA_ERR_OUT_OF_RANGE
 * and nothing is launched.  Every call on a GPU, from any context, uses that GPU's one array:
 * calls that overlap in time on one GPU race (serialise them on one stream); nothing in the array
 * needs clearing between calls, every share is written before it is read.                      */
ca_status ca_cached_prefill_attn_static(ca_ctx *ctx, int32_t layer, const void *q, const void *k_pool,
                                        const void *v_pool, void *out, float softmax_scale, void *stream);

/* ---- Section 3.2.2: asynchronous saving --------------------------------------------------- */
/* Copies context tokens [tok_begin[c], tok_end[c]) of every conversation (host int32 arrays;
 * NULL means the new tokens [n_keep, n_keep+new_len)) out of the pools into dst_k[c] / dst_v[c]
 * (contiguous layout, pointer to saved token 0) starting at token dst_tok_offset[c] (host int64
 * array; NULL means hist_len[c], i.e. append behind the saved history).  Keys leave without
 * positional encoding, exactly as stored.  Runs on the internal save stream after the work
 * queued so far on `after_stream`.  Destinations: device memory (written in place by the pack
 * kernel) or pinned host memory (pack kernel into a ring slot + hipMemcpyAsync, or written in place:
 * see save_mode).                                                                                  */
ca_status ca_kv_save_layer(ca_ctx *ctx, int32_t layer, const int32_t *tok_begin,
                           const int32_t *tok_end, const void *k_pool, const void *v_pool,
                           void *const *dst_k, void *const *dst_v, const int64_t *dst_tok_offset,
                           void *after_stream);

/* ca_kv_append_layer and ca_kv_save_layer (default range and offset: the new tokens go behind the
 * saved history of every conversation) in one call that reads new_k / new_v once: what is saved IS
 * what is appended, keys without positional encoding (Sections 3.2.2, 3.4), so the pool is not read
 * back.  Device destinations (and pinned ones under save_mode 2): one kernel on `stream` stores every
 * vector twice, to its page and to its row of the tier.  Pinned destinations otherwise: the append
 * kernel runs on `stream`; then either one copy per conversation follows on the internal save stream
 * straight from new_k / new_v (no pack kernel, no staging slot; new_k / new_v must then stay unchanged
 * until ca_sync or ca_join), or the pack kernel follows there and writes the tier in place (see
 * save_mode for which).  Same arguments, checks and statuses as the two calls it replaces.          */
ca_status ca_kv_append_save_layer(ca_ctx *ctx, int32_t layer, const void *new_k, const void *new_v,
                                  void *k_pool, void *v_pool, void *const *dst_k, void *const *dst_v,
                                  void *stream);

/* Blocks the host until the internal streams are idle. */
ca_status ca_sync(ca_ctx *ctx);

/* Makes `stream` wait (device side) for everything queued so far on the internal streams. */
ca_status ca_join(ca_ctx *ctx, void *stream);

/* ---- timing of the library's own GPU work ------------------------------------------------ */
/* While enabled, every copy batch and kernel the library queues is bracketed by HIP events on
 * the stream it runs on (the internal streams are not visible to the caller's own events).
 * ca_profile_read synchronises the device, returns the summed milliseconds and the number of
 * intervals of one kind recorded since the last read of that kind, and forgets them.
 * kind: 0 load copy-in (one interval per layer), 1 unpack kernel(s), 2 append kernel(s),
 *       3 attention kernel, 4 pack kernel(s), 5 save copy-out (one interval per layer).
 * on: 0 off; 1 every kind; any other value 2 * mask times only the kinds k with bit k of mask
 *     set (events cost a few per cent of a step of short kernels; a caller that needs one
 *     kernel's duration inside a timed region can restrict them to that kind).                 */
ca_status ca_profile_enable(ca_ctx *ctx, int32_t on);
ca_status ca_profile_read(ca_ctx *ctx, int32_t kind, double *total_ms, int64_t *count);

/* The recorded intervals that have not been read yet, in the order they were queued, without
 * forgetting them: kinds[i] as above, start_ms[i] and stop_ms[i] on one clock whose zero is the
 * start of the first interval still held (intervals of different streams are comparable, so the
 * overlap of copies and kernels can be read off). Host arrays of `capacity` entries each;
 * *count receives the number held, of which the first min(*count, capacity) are written.
 * Synchronises the device.                                                                   */
ca_status ca_profile_timeline(ca_ctx *ctx, int32_t *kinds, double *start_ms, double *stop_ms,
                              int64_t capacity, int64_t *count);

#ifdef __cplusplus
}
#endif
#endif /* CA_H_ */
