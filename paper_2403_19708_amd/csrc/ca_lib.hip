// Host side of the C ABI declared in include/ca.h: argument validation, the context (streams,
// events, staging ring, rotary table, plan metadata) and the stream choreography of the
// layer-wise load / save pipeline (Section 3.2).  Every step of the path itself runs in the
// kernels of ca_move.hip and ca_attn_*.hip; nothing here computes on the CPU except prefix
// sums over the batch (a few dozen integers) and the one-time rotary table.
#include "../../include/ca.h"
#include "ca_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <functional>
#include <new>
#include <string>
#include <vector>

using namespace ca;

// Partial-result buffer of ca_cached_prefill_attn_static: lives in the code object (one copy per GPU the library
// runs on, held until the process ends), so that entry point needs no allocation anywhere.  The name below is a
// host-side stand-in, not a device address: host code uses the per-device pointer that hipGetSymbolAddress
// returned (static_scratch_ptr), never the array itself.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) uint8_t scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void *static_scratch_ptr[kMaxDevices] = {nullptr};   // [device ordinal], filled by ca_create with that device current

struct ca_ctx {
    ca_config cfg{};
    hipStream_t s_copy = nullptr, s_unpack = nullptr, s_save = nullptr;
    // staging ring: `depth` slots for loads, `depth` for saves; slot = [K tokens | V tokens]
    uint8_t *load_slots = nullptr, *save_slots = nullptr;
    size_t slot_bytes = 0, half_slot_bytes = 0;
    std::vector<hipEvent_t> ev_slot_copied, ev_slot_copied2, ev_slot_free;  // per load slot
    std::vector<uint8_t> slot_used;
    int64_t load_count = 0, save_count = 0;
    float2 *rope = nullptr;
    // plan metadata: one pinned host image, one device image
    uint8_t *h_meta = nullptr, *d_meta = nullptr;
    size_t meta_bytes = 0;
    hipEvent_t ev_meta_copied = nullptr, ev_plan = nullptr, ev_after = nullptr;
    hipEvent_t ev_join[3] = {nullptr, nullptr, nullptr};
    bool meta_in_flight = false;
    // offsets (bytes) inside the metadata image
    size_t off_table = 0, off_n_keep = 0, off_cu_q = 0, off_cu_k = 0, off_items = 0, off_combine = 0, off_q_pos = 0,
           off_q_seq = 0, off_slot_map = 0, upload_bytes = 0;
    size_t items_capacity = 0;         // work items the image has room for
    float *partial = nullptr;          // shares of row tiles whose keys were split over workgroups
    uint16_t *k_rot = nullptr;         // keys of the batch context rotated once per layer (dense pages)
    uint16_t *v_t = nullptr;           // values of the batch context transposed once per layer (same pages)
    bool pipelined = false;             // the plan runs the software-pipelined kernel on the two scratch copies
    size_t off_rot_nvalid = 0;
    size_t k_rot_pages = 0;
    size_t off_dense0 = 0, off_rot_src = 0, off_rot_pos = 0;
    int32_t n_dense_pages = 0;
    bool prerotate = false;
    int32_t n_cus = 256;               // compute units of the device (balancing target)
    // current plan (host copies)
    bool has_plan = false;
    int32_t n_seqs = 0, max_pages = 0, num_pages = 0, n_items = 0, n_combine = 0, tile_rows = 128;
    int32_t max_unit_rows = 0;   // most stacked query rows of any (conversation, kv head) of the plan
    int32_t n_split_parts = 0;   // shares of split row tiles of the plan (slots of the partial-result buffer in use)
    float *static_partial = nullptr;   // this device's copy of the static scratch array (ca_cached_prefill_attn_static)
    int64_t total_q = 0, total_k = 0, total_n = 0;
    std::vector<int32_t> hist_len, new_len, n_keep, cu_q, cu_k;
    // kept saved tokens of conversation i: ranges keep_rng[keep_rng_at[i] .. keep_rng_at[i+1]) of (begin, end)
    std::vector<int32_t> keep_rng_at;
    std::vector<std::pair<int32_t, int32_t>> keep_rng;
    std::vector<int64_t> cu_n;
    std::vector<hipEvent_t> ev_ready;  // per layer
    std::vector<uint8_t> loaded;
    // optional timing of the library's own GPU work (ca_profile_*)
    struct Interval { int32_t kind; hipEvent_t start, stop; };
    bool profiling = false;
    uint32_t profile_mask = ~0u;       // bit k: intervals of kind k are recorded
    std::vector<Interval> intervals;
    std::vector<hipEvent_t> spare_events;
    std::string err;
};

namespace {

void set_err(char *dst, int32_t len, const char *fmt, ...) {
    if (!dst || len <= 0) return;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, (size_t)len, fmt, ap);
    va_end(ap);
}

ca_status fail(ca_ctx *ctx, ca_status st, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = buf;
    return st;
}

#define CA_HIP(ctx, expr)                                                                        \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess) {                                                                  \
            (void)hipGetLastError();                                                             \
            return fail((ctx), CA_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));      \
        }                                                                                        \
    } while (0)

constexpr int kHostStoreWorkgroups = 128;   // workgroups of a pack kernel whose destination is pinned host memory

// How a save reaches a pinned tier when the configuration leaves the choice to the library (save_mode 0).  Measured on
// MI355X with 64 conversations per layer: the per-conversation copies out of a staging slot (a few hundred KB each)
// move about 8 GB/s, run on a copy engine and disturb nothing; a pack kernel that stores over the host link moves about
// 40 GB/s, but while it runs an attention kernel beside it takes about that much longer (the slow stores hold up the
// queues its own stores go through).  The copies are the better choice as long as they hide under the layer's load
// (about 50 GB/s): fewer than a fifth as many tokens to save as kept history to load.  Beyond that the save stream
// would bound the step, and the kernel's bounded cost is the smaller one.
bool host_save_in_place(const ca_ctx *ctx, int64_t tokens_to_save) {
    if (ctx->cfg.save_mode != 0) return ctx->cfg.save_mode == 2;
    return tokens_to_save * 5 > ctx->total_n;
}

enum ProfileKind { kProfCopyIn = 0, kProfUnpack = 1, kProfAppend = 2, kProfAttn = 3, kProfPack = 4, kProfCopyOut = 5, kProfKinds = 6 };

hipError_t prof_event(ca_ctx *ctx, hipEvent_t *ev) {
    if (!ctx->spare_events.empty()) {
        *ev = ctx->spare_events.back();
        ctx->spare_events.pop_back();
        return hipSuccess;
    }
    return hipEventCreate(ev);
}

// Opens a timed interval on `stream`; returns its index or -1 when profiling is off.
hipError_t prof_begin(ca_ctx *ctx, int kind, hipStream_t stream, int *idx) {
    *idx = -1;
    if (!ctx->profiling || !(ctx->profile_mask & (1u << kind))) return hipSuccess;
    ca_ctx::Interval iv{kind, nullptr, nullptr};
    hipError_t e = prof_event(ctx, &iv.start);
    if (e != hipSuccess) return e;
    e = prof_event(ctx, &iv.stop);
    if (e != hipSuccess) return e;
    e = hipEventRecord(iv.start, stream);
    if (e != hipSuccess) return e;
    ctx->intervals.push_back(iv);
    *idx = (int)ctx->intervals.size() - 1;
    return hipSuccess;
}

hipError_t prof_end(ca_ctx *ctx, int idx, hipStream_t stream) {
    if (idx < 0) return hipSuccess;
    return hipEventRecord(ctx->intervals[idx].stop, stream);
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int64_t row_bytes(const ca_config &c) { return (int64_t)c.n_kv_heads * c.head_dim * 2; }

enum class MemKind { kDevice, kPinnedHost, kUnknown };

MemKind mem_kind(const void *p) {
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return MemKind::kUnknown;
    }
    if (attr.type == hipMemoryTypeDevice) return MemKind::kDevice;
    if (attr.type == hipMemoryTypeHost) return MemKind::kPinnedHost;
    if (attr.type == hipMemoryTypeManaged) return MemKind::kDevice;
    return MemKind::kUnknown;
}

// true if [p, p+bytes) lies inside one device allocation
bool device_range_ok(const void *p, size_t bytes) {
    if (!p) return false;
    if (mem_kind(p) != MemKind::kDevice) return false;
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    hipError_t e = hipMemGetAddressRange(&base, &size, (hipDeviceptr_t)p);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return true;  // kind was device; range query unsupported for this allocation
    }
    const uint8_t *b = (const uint8_t *)base, *q = (const uint8_t *)p;
    return q >= b && q + bytes <= b + size;
}

}  // namespace

extern "C" {

const char *ca_status_string(ca_status s) {
    switch (s) {
        case CA_OK: return "CA_OK";
        case CA_ERR_INVALID_ARG: return "CA_ERR_INVALID_ARG";
        case CA_ERR_OUT_OF_RANGE: return "CA_ERR_OUT_OF_RANGE";
        case CA_ERR_UNSUPPORTED: return "CA_ERR_UNSUPPORTED";
        case CA_ERR_NOMEM: return "CA_ERR_NOMEM";
        case CA_ERR_NOT_READY: return "CA_ERR_NOT_READY";
        case CA_ERR_HIP: return "CA_ERR_HIP";
    }
    return "CA_ERR_?";
}

void ca_config_default(ca_config *c) {
    if (!c) return;
    std::memset(c, 0, sizeof *c);
    c->n_layers = 1;
    c->n_q_heads = c->n_kv_heads = 1;
    c->head_dim = 128;
    c->page_size = kPageSize;
    c->max_positions = 4096;
    c->rope_base = 10000.0f;
    c->rope_style = 0;
    c->pipeline_depth = 2;
    c->max_seqs = 64;
    c->max_batch_kv_tokens = 1 << 16;
    c->max_batch_q_tokens = 1 << 14;
    c->load_mode = 0;
    c->save_mode = 0;
    c->attn_variant = 0;
    c->attn_tile_rows = 0;
    c->attn_split = 0;
    c->attn_prerotate = 0;
    c->attn_schedule = 0;
    c->require_load = 1;
    c->device = 0;
}

ca_status ca_config_validate(const ca_config *c, char *err, int32_t err_len) {
    if (!c) { set_err(err, err_len, "config is NULL"); return CA_ERR_INVALID_ARG; }
    if (c->n_layers < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1) {
        set_err(err, err_len, "n_layers, n_q_heads, n_kv_heads must be >= 1");
        return CA_ERR_INVALID_ARG;
    }
    if (c->n_q_heads % c->n_kv_heads != 0) {
        set_err(err, err_len, "n_q_heads (%d) is not a multiple of n_kv_heads (%d)", c->n_q_heads, c->n_kv_heads);
        return CA_ERR_INVALID_ARG;
    }
    if (c->head_dim != 64 && c->head_dim != 128) {
        set_err(err, err_len, "head_dim %d unsupported (64 or 128)", c->head_dim);
        return CA_ERR_UNSUPPORTED;
    }
    if (c->page_size != kPageSize) {
        set_err(err, err_len, "page_size %d unsupported (%d)", c->page_size, kPageSize);
        return CA_ERR_UNSUPPORTED;
    }
    if (c->rope_style != 0 && c->rope_style != 1) {
        set_err(err, err_len, "rope_style %d unsupported (0 or 1)", c->rope_style);
        return CA_ERR_UNSUPPORTED;
    }
    if (!(c->rope_base > 1.0f) || !std::isfinite(c->rope_base)) {
        set_err(err, err_len, "rope_base must be finite and > 1");
        return CA_ERR_INVALID_ARG;
    }
    if (c->max_positions < 1 || c->max_positions > (1 << 20)) {
        set_err(err, err_len, "max_positions %d out of range [1, 2^20]", c->max_positions);
        return CA_ERR_OUT_OF_RANGE;
    }
    if (c->pipeline_depth < 1 || c->pipeline_depth > 64) {
        set_err(err, err_len, "pipeline_depth %d out of range [1, 64]", c->pipeline_depth);
        return CA_ERR_OUT_OF_RANGE;
    }
    if (c->max_seqs < 1 || c->max_seqs > 4096) {
        set_err(err, err_len, "max_seqs %d out of range [1, 4096]", c->max_seqs);
        return CA_ERR_OUT_OF_RANGE;
    }
    if (c->max_batch_kv_tokens < 1 || c->max_batch_kv_tokens > ((int64_t)1 << 26) ||
        c->max_batch_q_tokens < 1 || c->max_batch_q_tokens > c->max_batch_kv_tokens) {
        set_err(err, err_len, "max_batch_kv_tokens / max_batch_q_tokens out of range");
        return CA_ERR_OUT_OF_RANGE;
    }
    if (c->save_mode < 0 || c->save_mode > 2) {
        set_err(err, err_len, "save_mode (0..2) out of range");
        return CA_ERR_INVALID_ARG;
    }
    if (c->load_mode < 0 || c->load_mode > 2 || c->attn_variant < 0 || c->attn_variant > 4) {
        set_err(err, err_len, "load_mode (0..2) or attn_variant (0..4) out of range");
        return CA_ERR_INVALID_ARG;
    }
    if (c->attn_variant == 3) {
        set_err(err, err_len, "attn_variant 3 (the register-staged kernel) was removed: the LDS-direct kernel serves every window");
        return CA_ERR_UNSUPPORTED;
    }
    if (c->attn_tile_rows != 0 && c->attn_tile_rows != 128 && c->attn_tile_rows != 256) {
        set_err(err, err_len, "attn_tile_rows %d unsupported (0, 128 or 256)", c->attn_tile_rows);
        return CA_ERR_UNSUPPORTED;
    }
    if (c->attn_prerotate < 0 || c->attn_prerotate > 2) { set_err(err, err_len, "attn_prerotate must be 0, 1 or 2"); return CA_ERR_INVALID_ARG; }
    if (c->attn_schedule < 0 || c->attn_schedule > 1) { set_err(err, err_len, "attn_schedule must be 0 or 1"); return CA_ERR_INVALID_ARG; }
    if (c->attn_split < 0 || c->attn_split > 1) { set_err(err, err_len, "attn_split must be 0 or 1"); return CA_ERR_INVALID_ARG; }
    if (c->device < 0) { set_err(err, err_len, "device < 0"); return CA_ERR_INVALID_ARG; }
    return CA_OK;
}

ca_status ca_batch_validate(const ca_config *c, const ca_batch *b, char *err, int32_t err_len) {
    ca_status st = ca_config_validate(c, err, err_len);
    if (st != CA_OK) return st;
    if (!b || !b->hist_len || !b->new_len || !b->block_table) {
        set_err(err, err_len, "batch or one of its arrays is NULL");
        return CA_ERR_INVALID_ARG;
    }
    if ((b->keep_ranges == nullptr) != (b->keep_range_count == nullptr)) {
        set_err(err, err_len, "keep_ranges and keep_range_count must both be given or both NULL");
        return CA_ERR_INVALID_ARG;
    }
    if (!b->keep_ranges && !b->keep_start) {
        set_err(err, err_len, "neither keep_start nor keep_ranges is given");
        return CA_ERR_INVALID_ARG;
    }
    if (b->n_seqs < 1 || b->n_seqs > c->max_seqs) {
        set_err(err, err_len, "n_seqs %d out of range [1, max_seqs=%d]", b->n_seqs, c->max_seqs);
        return CA_ERR_OUT_OF_RANGE;
    }
    if (b->max_pages < 1 || b->num_pages < 1) {
        set_err(err, err_len, "max_pages and num_pages must be >= 1");
        return CA_ERR_INVALID_ARG;
    }
    if ((int64_t)b->num_pages * c->page_size > ((int64_t)1 << 31) - 1) {
        set_err(err, err_len, "num_pages %d: slot index would overflow int32", b->num_pages);
        return CA_ERR_OUT_OF_RANGE;
    }
    int64_t tot_k = 0, tot_q = 0, range_at = 0;
    std::vector<uint8_t> seen((size_t)b->num_pages, 0);
    for (int32_t i = 0; i < b->n_seqs; ++i) {
        const int64_t h = b->hist_len[i], n = b->new_len[i];
        if (h < 0 || n < 1) {
            set_err(err, err_len, "conversation %d: hist_len %lld < 0 or new_len %lld < 1", i, (long long)h, (long long)n);
            return CA_ERR_INVALID_ARG;
        }
        int64_t kept = 0;
        if (b->keep_ranges) {
            const int64_t cnt = b->keep_range_count[i];
            if (cnt < 0 || cnt > h) {
                set_err(err, err_len, "conversation %d: keep_range_count %lld outside [0, hist_len=%lld]", i, (long long)cnt, (long long)h);
                return CA_ERR_OUT_OF_RANGE;
            }
            int64_t prev_end = 0;
            for (int64_t r = 0; r < cnt; ++r) {
                const int64_t rb = b->keep_ranges[2 * (range_at + r)], re = b->keep_ranges[2 * (range_at + r) + 1];
                if (rb < prev_end || re <= rb || re > h) {
                    set_err(err, err_len, "conversation %d: kept range %lld = [%lld, %lld) is empty, out of order or outside [0, hist_len=%lld]",
                            i, (long long)r, (long long)rb, (long long)re, (long long)h);
                    return CA_ERR_OUT_OF_RANGE;
                }
                kept += re - rb;
                prev_end = re;
            }
            range_at += cnt;
        } else {
            const int64_t s = b->keep_start[i];
            if (s < 0 || s > h) {
                set_err(err, err_len, "conversation %d: keep_start %lld outside [0, hist_len=%lld]", i, (long long)s, (long long)h);
                return CA_ERR_OUT_OF_RANGE;
            }
            kept = h - s;
        }
        const int64_t ctx_len = kept + n;
        if (ctx_len > c->max_positions) {
            set_err(err, err_len, "conversation %d: context %lld exceeds max_positions %d (truncate first)", i,
                    (long long)ctx_len, c->max_positions);
            return CA_ERR_OUT_OF_RANGE;
        }
        const int64_t pages = (ctx_len + c->page_size - 1) / c->page_size;
        if (pages > b->max_pages) {
            set_err(err, err_len, "conversation %d: needs %lld pages, block table has %d columns", i, (long long)pages, b->max_pages);
            return CA_ERR_OUT_OF_RANGE;
        }
        for (int64_t p = 0; p < pages; ++p) {
            const int32_t page = b->block_table[(int64_t)i * b->max_pages + p];
            if (page < 0 || page >= b->num_pages) {
                set_err(err, err_len, "conversation %d: block_table[%lld] = %d outside [0, num_pages=%d)", i, (long long)p, page, b->num_pages);
                return CA_ERR_OUT_OF_RANGE;
            }
            if (seen[(size_t)page]) {
                set_err(err, err_len, "conversation %d: page %d is used twice in the batch", i, page);
                return CA_ERR_INVALID_ARG;
            }
            seen[(size_t)page] = 1;
        }
        tot_k += ctx_len;
        tot_q += n;
    }
    if (tot_k > c->max_batch_kv_tokens || tot_q > c->max_batch_q_tokens) {
        set_err(err, err_len, "batch has %lld context / %lld new tokens, limits are %lld / %lld", (long long)tot_k,
                (long long)tot_q, (long long)c->max_batch_kv_tokens, (long long)c->max_batch_q_tokens);
        return CA_ERR_OUT_OF_RANGE;
    }
    return CA_OK;
}

ca_status ca_truncate_plan_sinks(const int32_t *hist_len, const int32_t *new_len, int32_t window, double ratio,
                                 int32_t n_sink, int32_t n, int32_t *ranges_out, int32_t *count_out) {
    if (!hist_len || !new_len || !ranges_out || !count_out || n < 0 || n_sink < 0) return CA_ERR_INVALID_ARG;
    if (window < 1 || !(ratio > 0.0) || !(ratio < 1.0)) return CA_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i)
        if (hist_len[i] < 0 || new_len[i] < 0) return CA_ERR_INVALID_ARG;
    const int64_t keep_target = (int64_t)std::floor((double)window * (1.0 - ratio));
    for (int32_t i = 0; i < n; ++i) {
        const int64_t h = hist_len[i], fresh = new_len[i];
        int32_t *r = ranges_out + 4 * (int64_t)i;
        r[0] = r[1] = r[2] = r[3] = 0;
        int32_t cnt = 0;
        if (h + fresh <= window) {
            if (h > 0) { r[0] = 0; r[1] = (int32_t)h; cnt = 1; }
        } else {
            const int64_t budget = std::min<int64_t>(h, std::max<int64_t>(0, keep_target - fresh));
            const int64_t sinks = std::min<int64_t>(n_sink, budget);
            const int64_t recent = budget - sinks;                 // tokens [h - recent, h)
            if (sinks > 0 && recent > 0 && h - recent <= sinks) {  // the two pieces touch or overlap
                r[0] = 0; r[1] = (int32_t)h; cnt = 1;              // (only when everything is kept)
            } else {
                if (sinks > 0) { r[2 * cnt] = 0; r[2 * cnt + 1] = (int32_t)sinks; ++cnt; }
                if (recent > 0) { r[2 * cnt] = (int32_t)(h - recent); r[2 * cnt + 1] = (int32_t)h; ++cnt; }
            }
        }
        count_out[i] = cnt;
    }
    return CA_OK;
}

ca_status ca_tier_compact(int32_t n, const int32_t *hist_len, const int32_t *keep_start, const int32_t *keep_ranges,
                          const int32_t *keep_range_count, int64_t row_bytes, void *const *tier_k, void *const *tier_v,
                          int32_t *hist_len_out) {
    if (n < 0 || !hist_len || !tier_k || !tier_v || !hist_len_out || row_bytes <= 0) return CA_ERR_INVALID_ARG;
    if ((keep_ranges == nullptr) != (keep_range_count == nullptr)) return CA_ERR_INVALID_ARG;
    if (!keep_ranges && !keep_start) return CA_ERR_INVALID_ARG;
    // everything is checked before the first byte moves
    int64_t at = 0;
    for (int32_t c = 0; c < n; ++c) {
        if (hist_len[c] < 0) return CA_ERR_INVALID_ARG;
        if (keep_ranges) {
            if (keep_range_count[c] < 0) return CA_ERR_INVALID_ARG;
            int32_t prev_end = 0;
            for (int32_t r = 0; r < keep_range_count[c]; ++r, ++at) {
                const int32_t b = keep_ranges[2 * at], e = keep_ranges[2 * at + 1];
                if (b < prev_end || e <= b || e > hist_len[c]) return CA_ERR_OUT_OF_RANGE;
                prev_end = e;
            }
            if (keep_range_count[c] > 0 && (!tier_k[c] || !tier_v[c])) return CA_ERR_INVALID_ARG;
        } else {
            if (keep_start[c] < 0 || keep_start[c] > hist_len[c]) return CA_ERR_OUT_OF_RANGE;
            if (keep_start[c] < hist_len[c] && (!tier_k[c] || !tier_v[c])) return CA_ERR_INVALID_ARG;
        }
    }
    at = 0;
    for (int32_t c = 0; c < n; ++c) {
        int64_t dst = 0;   // rows written so far; a range never starts below it, so the moves go towards lower addresses
        auto move = [&](int32_t b, int32_t e) {
            const size_t bytes = (size_t)(e - b) * (size_t)row_bytes;
            if (b != dst) {
                std::memmove((uint8_t *)tier_k[c] + (size_t)dst * row_bytes, (const uint8_t *)tier_k[c] + (size_t)b * row_bytes, bytes);
                std::memmove((uint8_t *)tier_v[c] + (size_t)dst * row_bytes, (const uint8_t *)tier_v[c] + (size_t)b * row_bytes, bytes);
            }
            dst += e - b;
        };
        if (keep_ranges) {
            for (int32_t r = 0; r < keep_range_count[c]; ++r, ++at) move(keep_ranges[2 * at], keep_ranges[2 * at + 1]);
        } else if (keep_start[c] < hist_len[c]) {
            move(keep_start[c], hist_len[c]);
        }
        hist_len_out[c] = (int32_t)dst;
    }
    return CA_OK;
}

ca_status ca_truncate_plan(const int32_t *hist_len, const int32_t *new_len, int32_t window, double ratio,
                           int32_t policy, int32_t n, int32_t *keep_start_out) {
    if (!hist_len || !new_len || !keep_start_out || n < 0) return CA_ERR_INVALID_ARG;
    if (window < 1 || !(ratio > 0.0) || !(ratio < 1.0)) return CA_ERR_INVALID_ARG;
    if (policy < 0 || policy > 2) return CA_ERR_UNSUPPORTED;
    for (int32_t i = 0; i < n; ++i)
        if (hist_len[i] < 0 || new_len[i] < 0) return CA_ERR_INVALID_ARG;
    const int64_t keep_target = (int64_t)std::floor((double)window * (1.0 - ratio));
    const int64_t drop_fixed = std::max<int64_t>(1, (int64_t)std::floor((double)window * ratio));
    for (int32_t i = 0; i < n; ++i) {
        const int64_t h = hist_len[i], fresh = new_len[i];
        int64_t first = 0;  // first surviving history token
        if (h + fresh > window) {
            switch (policy) {
                case 0:
                    first = h - std::min(h, std::max<int64_t>(0, keep_target - fresh));
                    break;
                case 1:
                    while (first < h && h - first + fresh > window) first = std::min(h, first + drop_fixed);
                    break;
                default:
                    while (first < h && h - first + fresh > window) {
                        const int64_t d = (int64_t)std::floor(ratio * (double)(h - first + fresh));
                        first = std::min(h, first + std::max<int64_t>(1, d));
                    }
            }
        }
        keep_start_out[i] = (int32_t)first;
    }
    return CA_OK;
}

const char *ca_last_error(const ca_ctx *ctx) { return ctx ? ctx->err.c_str() : "context is NULL"; }

void ca_destroy(ca_ctx *ctx) {
    if (!ctx) return;
    (void)hipSetDevice(ctx->cfg.device);
    if (ctx->s_copy) (void)hipStreamSynchronize(ctx->s_copy);
    if (ctx->s_unpack) (void)hipStreamSynchronize(ctx->s_unpack);
    if (ctx->s_save) (void)hipStreamSynchronize(ctx->s_save);
    for (auto e : ctx->ev_slot_copied) if (e) (void)hipEventDestroy(e);
    for (auto e : ctx->ev_slot_copied2) if (e) (void)hipEventDestroy(e);
    for (auto e : ctx->ev_slot_free) if (e) (void)hipEventDestroy(e);
    for (auto e : ctx->ev_ready) if (e) (void)hipEventDestroy(e);
    if (ctx->ev_meta_copied) (void)hipEventDestroy(ctx->ev_meta_copied);
    if (ctx->ev_plan) (void)hipEventDestroy(ctx->ev_plan);
    if (ctx->ev_after) (void)hipEventDestroy(ctx->ev_after);
    for (auto e : ctx->ev_join) if (e) (void)hipEventDestroy(e);
    for (auto &iv : ctx->intervals) { (void)hipEventDestroy(iv.start); (void)hipEventDestroy(iv.stop); }
    for (auto e : ctx->spare_events) (void)hipEventDestroy(e);
    if (ctx->load_slots) (void)hipFree(ctx->load_slots);
    if (ctx->save_slots) (void)hipFree(ctx->save_slots);
    if (ctx->rope) (void)hipFree(ctx->rope);
    if (ctx->partial) (void)hipFree(ctx->partial);
    if (ctx->k_rot) (void)hipFree(ctx->k_rot);
    if (ctx->v_t) (void)hipFree(ctx->v_t);
    if (ctx->d_meta) (void)hipFree(ctx->d_meta);
    if (ctx->h_meta) (void)hipHostFree(ctx->h_meta);
    if (ctx->s_copy) (void)hipStreamDestroy(ctx->s_copy);
    if (ctx->s_unpack) (void)hipStreamDestroy(ctx->s_unpack);
    if (ctx->s_save) (void)hipStreamDestroy(ctx->s_save);
    delete ctx;
}

// every variant but the scalar check kernel stages K/V through LDS without registers (any window: the kernels keep a
// moving window of page ids in LDS)
static bool direct_variant(const ca_config &c) { return c.attn_variant != 1; }

static ca_status create_impl(ca_ctx *ctx) {
    const ca_config &c = ctx->cfg;
    int n_dev = 0;
    CA_HIP(ctx, hipGetDeviceCount(&n_dev));
    if (c.device >= n_dev) return fail(ctx, CA_ERR_OUT_OF_RANGE, "device %d of %d", c.device, n_dev);
    CA_HIP(ctx, hipSetDevice(c.device));
    CA_HIP(ctx, hipStreamCreateWithFlags(&ctx->s_copy, hipStreamNonBlocking));
    CA_HIP(ctx, hipStreamCreateWithFlags(&ctx->s_unpack, hipStreamNonBlocking));
    CA_HIP(ctx, hipStreamCreateWithFlags(&ctx->s_save, hipStreamNonBlocking));
    const int depth = c.pipeline_depth;
    ctx->half_slot_bytes = align_up((size_t)c.max_batch_kv_tokens * (size_t)row_bytes(c), 256);
    ctx->slot_bytes = 2 * ctx->half_slot_bytes;
    CA_HIP(ctx, hipMalloc((void **)&ctx->load_slots, ctx->slot_bytes * depth));
    CA_HIP(ctx, hipMalloc((void **)&ctx->save_slots, ctx->slot_bytes * depth));
    ctx->ev_slot_copied.assign(depth, nullptr);
    ctx->ev_slot_copied2.assign(depth, nullptr);
    ctx->ev_slot_free.assign(depth, nullptr);
    ctx->slot_used.assign(depth, 0);
    for (int i = 0; i < depth; ++i) {
        CA_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_slot_copied[i], hipEventDisableTiming));
        CA_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_slot_copied2[i], hipEventDisableTiming));
        CA_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_slot_free[i], hipEventDisableTiming));
    }
    ctx->ev_ready.assign(c.n_layers, nullptr);
    ctx->loaded.assign(c.n_layers, 0);
    for (int i = 0; i < c.n_layers; ++i)
        CA_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_ready[i], hipEventDisableTiming));
    CA_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_meta_copied, hipEventDisableTiming));
    CA_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_plan, hipEventDisableTiming));
    CA_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_after, hipEventDisableTiming));
    for (auto &e : ctx->ev_join) CA_HIP(ctx, hipEventCreateWithFlags(&e, hipEventDisableTiming));

    // Rotary table (Section 3.4): cos/sin of pos * base^(-2i/D), evaluated in fp64, stored fp32.
    {
        const int half = c.head_dim / 2;
        const int rows = std::max(c.max_positions, kRopeMinRows);
        std::vector<float2> tab((size_t)rows * half);
        std::vector<double> inv_freq(half);
        for (int i = 0; i < half; ++i)
            inv_freq[i] = std::exp(-std::log((double)c.rope_base) * (2.0 * i) / (double)c.head_dim);
        for (int p = 0; p < rows; ++p)
            for (int i = 0; i < half; ++i) {
                const double ang = (double)p * inv_freq[i];
                tab[(size_t)p * half + i] = make_float2((float)std::cos(ang), (float)std::sin(ang));
            }
        CA_HIP(ctx, hipMalloc((void **)&ctx->rope, tab.size() * sizeof(float2)));
        CA_HIP(ctx, hipMemcpy(ctx->rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice));
    }

    // Metadata image layout.  Uploaded part first (block table rows are packed to the batch's
    // max_pages, bounded by ceil(max_positions/page)+1 columns), device-computed arrays after it.
    {
        const size_t max_cols = (size_t)(c.max_positions + c.page_size - 1) / c.page_size + 1;
        const size_t units = (size_t)c.max_seqs * c.n_kv_heads;
        const size_t g = (size_t)c.n_q_heads / c.n_kv_heads;
        // tiles: sum over units of ceil(rows/tile) <= total_q*g*n_kv_heads/tile + units, padded per die
        // (+ the extra items that splitting keys can add)
        const size_t max_items = (size_t)c.max_batch_q_tokens * g * c.n_kv_heads / kAttnTileRowsMin + units + kAttnMaxParts;
        const size_t max_items_padded = (max_items + 1) * kXcds;  // worst case: every tile on one die
        ctx->items_capacity = max_items_padded;
        size_t off = 0;
        ctx->off_table = off;   off = align_up(off + (size_t)c.max_seqs * max_cols * 4, 256);
        ctx->off_n_keep = off;  off = align_up(off + (size_t)c.max_seqs * 4, 256);
        ctx->off_cu_q = off;    off = align_up(off + ((size_t)c.max_seqs + 1) * 4, 256);
        ctx->off_cu_k = off;    off = align_up(off + ((size_t)c.max_seqs + 1) * 4, 256);
        ctx->k_rot_pages = (size_t)c.max_batch_kv_tokens / c.page_size + (size_t)c.max_seqs;
        ctx->off_dense0 = off;  off = align_up(off + (size_t)c.max_seqs * 4, 256);
        ctx->off_rot_src = off; off = align_up(off + ctx->k_rot_pages * 4, 256);
        ctx->off_rot_pos = off; off = align_up(off + ctx->k_rot_pages * 4, 256);
        ctx->off_rot_nvalid = off; off = align_up(off + ctx->k_rot_pages * 4, 256);
        ctx->off_combine = off; off = align_up(off + (size_t)kAttnMaxParts * sizeof(CombineItem), 256);
        ctx->off_items = off;   off = align_up(off + max_items_padded * sizeof(WorkItem), 256);
        ctx->upload_bytes = off;
        ctx->off_q_pos = off;   off = align_up(off + (size_t)c.max_batch_q_tokens * 4, 256);
        ctx->off_q_seq = off;   off = align_up(off + (size_t)c.max_batch_q_tokens * 4, 256);
        ctx->off_slot_map = off; off = align_up(off + (size_t)c.max_batch_kv_tokens * 4, 256);
        ctx->meta_bytes = off;
        CA_HIP(ctx, hipMalloc((void **)&ctx->d_meta, ctx->meta_bytes));
        CA_HIP(ctx, hipHostMalloc((void **)&ctx->h_meta, ctx->upload_bytes, hipHostMallocDefault));
    }
    // Partial results of row tiles whose keys are split over workgroups (only the LDS-direct kernel splits).
    const bool may_split = c.attn_split == 0 && direct_variant(c);
    if (may_split) {
        const size_t bytes = (size_t)kAttnMaxParts * 256 * (size_t)(c.head_dim + 2) * sizeof(float);
        CA_HIP(ctx, hipMalloc((void **)&ctx->partial, bytes));
    }
    const bool may_direct = direct_variant(c);
    if (may_direct && c.attn_prerotate != 1) {
        CA_HIP(ctx, hipMalloc((void **)&ctx->k_rot, ctx->k_rot_pages * (size_t)c.page_size * (size_t)row_bytes(c)));
        if (c.head_dim == 128 && c.attn_schedule == 1)
            CA_HIP(ctx, hipMalloc((void **)&ctx->v_t, ctx->k_rot_pages * (size_t)c.page_size * (size_t)row_bytes(c)));
    }
    {
        hipDeviceProp_t prop;
        CA_HIP(ctx, hipGetDeviceProperties(&prop, c.device));
        ctx->n_cus = std::max(8, prop.multiProcessorCount);
    }
    // address of this device's copy of the static scratch array (the device is current here)
    if (c.device < kMaxDevices) {
        if (!static_scratch_ptr[c.device]) {
            void *p = nullptr;
            CA_HIP(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            static_scratch_ptr[c.device] = p;
        }
        ctx->static_partial = (float *)static_scratch_ptr[c.device];
    }
    return CA_OK;
}

ca_status ca_create(const ca_config *cfg, ca_ctx **out) {
    if (!out) return CA_ERR_INVALID_ARG;
    *out = nullptr;
    char msg[256] = {0};
    ca_status st = ca_config_validate(cfg, msg, sizeof msg);
    if (st != CA_OK) return st;
    ca_ctx *ctx = new (std::nothrow) ca_ctx();
    if (!ctx) return CA_ERR_NOMEM;
    ctx->cfg = *cfg;
    st = create_impl(ctx);
    if (st != CA_OK) {
        if (st == CA_ERR_HIP && ctx->err.find("out of memory") != std::string::npos) st = CA_ERR_NOMEM;
        std::fprintf(stderr, "ca_create: %s\n", ctx->err.c_str());
        ca_destroy(ctx);
        return st;
    }
    *out = ctx;
    return CA_OK;
}

ca_status ca_sync(ca_ctx *ctx) {
    if (!ctx) return CA_ERR_INVALID_ARG;
    CA_HIP(ctx, hipStreamSynchronize(ctx->s_copy));
    CA_HIP(ctx, hipStreamSynchronize(ctx->s_unpack));
    CA_HIP(ctx, hipStreamSynchronize(ctx->s_save));
    return CA_OK;
}

ca_status ca_join(ca_ctx *ctx, void *stream) {
    if (!ctx) return CA_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    hipStream_t internal[3] = {ctx->s_copy, ctx->s_unpack, ctx->s_save};
    for (int i = 0; i < 3; ++i) {
        CA_HIP(ctx, hipEventRecord(ctx->ev_join[i], internal[i]));
        CA_HIP(ctx, hipStreamWaitEvent(s, ctx->ev_join[i], 0));
    }
    return CA_OK;
}

// ----------------------------------------------------------------------------------------------
// Section 3.4: rebase
// ----------------------------------------------------------------------------------------------
ca_status ca_rope_rebase(ca_ctx *ctx, const ca_batch *b, void *stream_) {
    if (!ctx) return CA_ERR_INVALID_ARG;
    char msg[384] = {0};
    ca_status st = ca_batch_validate(&ctx->cfg, b, msg, sizeof msg);
    if (st != CA_OK) return fail(ctx, st, "ca_rope_rebase: %s", msg);
    const ca_config &c = ctx->cfg;
    hipStream_t stream = (hipStream_t)stream_;
    CA_HIP(ctx, hipSetDevice(c.device));

    const int B = b->n_seqs;
    const size_t max_cols = (size_t)(c.max_positions + c.page_size - 1) / c.page_size + 1;
    const int cols = (int)std::min<size_t>((size_t)b->max_pages, max_cols);

    // the pinned image may still be the source of the previous plan's upload
    if (ctx->meta_in_flight) {
        CA_HIP(ctx, hipEventSynchronize(ctx->ev_meta_copied));
        ctx->meta_in_flight = false;
    }

    // from here on the host copy of the plan is rewritten: until the new metadata has been queued for upload
    // the context has no usable plan (a failure below must not leave new host counts beside old device tables)
    ctx->has_plan = false;
    ctx->hist_len.assign(b->hist_len, b->hist_len + B);
    ctx->keep_rng_at.assign(B + 1, 0);
    ctx->keep_rng.clear();
    for (int i = 0, at = 0; i < B; ++i) {
        if (b->keep_ranges) {
            for (int r = 0; r < b->keep_range_count[i]; ++r, ++at)
                ctx->keep_rng.push_back({b->keep_ranges[2 * at], b->keep_ranges[2 * at + 1]});
        } else if (b->keep_start[i] < b->hist_len[i]) {
            ctx->keep_rng.push_back({b->keep_start[i], b->hist_len[i]});
        }
        ctx->keep_rng_at[i + 1] = (int32_t)ctx->keep_rng.size();
    }
    ctx->new_len.assign(b->new_len, b->new_len + B);
    ctx->n_keep.resize(B);
    ctx->cu_q.assign(B + 1, 0);
    ctx->cu_k.assign(B + 1, 0);
    ctx->cu_n.assign(B + 1, 0);
    for (int i = 0; i < B; ++i) {
        int32_t kept = 0;
        for (int r = ctx->keep_rng_at[i]; r < ctx->keep_rng_at[i + 1]; ++r) kept += ctx->keep_rng[r].second - ctx->keep_rng[r].first;
        ctx->n_keep[i] = kept;
        ctx->cu_q[i + 1] = ctx->cu_q[i] + b->new_len[i];
        ctx->cu_k[i + 1] = ctx->cu_k[i] + ctx->n_keep[i] + b->new_len[i];
        ctx->cu_n[i + 1] = ctx->cu_n[i] + ctx->n_keep[i];
    }
    ctx->n_seqs = B;
    ctx->max_pages = cols;
    ctx->num_pages = b->num_pages;
    ctx->total_q = ctx->cu_q[B];
    ctx->total_k = ctx->cu_k[B];
    ctx->total_n = ctx->cu_n[B];

    // ---- host image -------------------------------------------------------------------------
    int32_t *h_table = (int32_t *)(ctx->h_meta + ctx->off_table);
    for (int i = 0; i < B; ++i) {
        const int64_t ctx_len = (int64_t)ctx->n_keep[i] + b->new_len[i];
        const int pages = (int)((ctx_len + c.page_size - 1) / c.page_size);
        for (int p = 0; p < cols; ++p)  // unused columns point at the row's first page: always a valid page
            h_table[(size_t)i * cols + p] = b->block_table[(int64_t)i * b->max_pages + (p < pages ? p : 0)];
    }
    std::memcpy(ctx->h_meta + ctx->off_n_keep, ctx->n_keep.data(), (size_t)B * 4);
    std::memcpy(ctx->h_meta + ctx->off_cu_q, ctx->cu_q.data(), (size_t)(B + 1) * 4);
    std::memcpy(ctx->h_meta + ctx->off_cu_k, ctx->cu_k.data(), (size_t)(B + 1) * 4);

    // ---- attention work list: tiles of stacked query rows, placed die by die ------------------
    // All tiles of one (conversation, kv head) read the same keys/values, so they are given to the
    // same die (workgroup i runs on die i % 8) in consecutive launch slots and share its L2.
    // Units go longest-first to the least loaded die; dies are padded to equal length.
    {
        const int G = c.n_q_heads / c.n_kv_heads;
        // 256-row tiles (8 wavefronts) halve the K/V re-reads and the rotary work per row when a
        // (conversation, kv head) has more than 128 stacked rows; small turns keep 128-row tiles
        int tile = c.attn_tile_rows;
        int most = 0;
        for (int i = 0; i < B; ++i) most = std::max(most, b->new_len[i] * G);
        ctx->max_unit_rows = most;
        if (tile == 0) tile = most > 128 ? 256 : 128;
        const bool direct_for_rot = direct_variant(c);
        {   // rotate the keys once per layer when on average three or more row tiles would each rotate them
            int64_t tiles256 = 0;
            for (int i = 0; i < B; ++i) tiles256 += ((int64_t)b->new_len[i] * G + 255) / 256;
            ctx->prerotate = ctx->k_rot && direct_for_rot &&
                             (c.attn_prerotate == 2 || (c.attn_prerotate == 0 && tiles256 >= (int64_t)3 * B));
            if (ctx->prerotate && c.attn_tile_rows == 0) tile = 256;
            ctx->pipelined = ctx->prerotate && ctx->v_t && tile == 256 && c.attn_variant != 3 && c.attn_variant != 1;
            int32_t *dense0 = (int32_t *)(ctx->h_meta + ctx->off_dense0);
            int32_t *rot_src = (int32_t *)(ctx->h_meta + ctx->off_rot_src), *rot_pos = (int32_t *)(ctx->h_meta + ctx->off_rot_pos);
            int32_t *rot_nvalid = (int32_t *)(ctx->h_meta + ctx->off_rot_nvalid);
            int32_t at = 0;
            for (int i = 0; i < B; ++i) {
                dense0[i] = at;
                if (!ctx->prerotate) continue;
                const int pages = (ctx->n_keep[i] + b->new_len[i] + c.page_size - 1) / c.page_size;
                for (int p = 0; p < pages; ++p, ++at) {
                    rot_src[at] = b->block_table[(int64_t)i * b->max_pages + p];
                    rot_pos[at] = p * c.page_size;
                    rot_nvalid[at] = std::min(c.page_size, ctx->n_keep[i] + b->new_len[i] - p * c.page_size);
                }
            }
            if ((size_t)at > ctx->k_rot_pages) return fail(ctx, CA_ERR_OUT_OF_RANGE, "ca_rope_rebase: internal: %d dense pages exceed %zu", at, ctx->k_rot_pages);
            ctx->n_dense_pages = at;
        }
        ctx->tile_rows = tile;
        const bool direct_kernel = direct_variant(c);
        struct Unit { int32_t seq, head; int64_t work; };
        std::vector<Unit> units;
        units.reserve((size_t)B * c.n_kv_heads);
        for (int i = 0; i < B; ++i) {
            const int64_t ln = b->new_len[i], n = ctx->n_keep[i];
            const int64_t work = (int64_t)G * (ln * n + ln * (ln + 1) / 2);
            for (int g = 0; g < c.n_kv_heads; ++g) units.push_back({i, g, work});
        }
        std::stable_sort(units.begin(), units.end(), [](const Unit &x, const Unit &y) { return x.work > y.work; });
        int64_t total_tiles = 0;
        for (const Unit &u : units) total_tiles += (b->new_len[u.seq] * G + tile - 1) / tile;
        // a unit with more tiles than a die's fair share is cut into chunks so that a small batch
        // still spreads over all dies
        const int chunk_cap = (int)std::max<int64_t>(1, (total_tiles + kXcds - 1) / kXcds);
        // Cost of an item in the time a full workgroup needs for one 64-key tile (measured on single items:
        // a 256-row workgroup whose rows fill at most four wavefronts, one per SIMD, takes 0.72 of that per
        // tile; rotating Q, filling the load pipeline and the epilogue cost about three tiles).
        struct Item { WorkItem w; double cost; int32_t parent; };
        // A plan of decode steps goes to the streaming kernel, which reaches its bandwidth with one workgroup
        // per compute unit: shares (and the merge they need) only pay when there are fewer items than that.
        const bool decode_plan = direct_kernel && c.attn_variant != 2 && !ctx->prerotate && most >= 1 && most <= kAttnDecodeMaxRows;
        auto item_cost = [&](int n_rows, int keys) {
            const double per_tile = (tile == 256 && n_rows <= 128) ? 0.72 : 1.0;
            return per_tile * ((keys + 63) / 64) + 3.0;
        };
        std::vector<std::vector<Item>> per_die(kXcds);
        double load[kXcds] = {0};
        int32_t n_parents = 0;
        for (const Unit &u : units) {
            const int rows = b->new_len[u.seq] * G;
            const int n_tiles = (rows + tile - 1) / tile;
            const int n = ctx->n_keep[u.seq];
            for (int hi = n_tiles; hi > 0; hi -= chunk_cap) {  // later rows see more keys: longest first
                const int lo = std::max(0, hi - chunk_cap);
                int die = 0;
                for (int d = 1; d < kXcds; ++d) if (load[d] < load[die]) die = d;
                for (int t = hi - 1; t >= lo; --t) {
                    const int n_rows = std::min(tile, rows - t * tile);
                    const int keys = n + (t * tile + n_rows - 1) / G + 1;       // what the tile's rows see
                    const double cost = item_cost(n_rows, keys);
                    load[die] += cost;
                    per_die[die].push_back({WorkItem{u.seq, u.head, t * tile, n_rows, 0, keys, -1, 0}, cost, n_parents++});
                }
            }
        }

        // Few, long items leave compute units idle at the end (or, for a small batch, from the start): split
        // the keys of the longest items over several workgroups until a longest-first schedule of the die's
        // items over its compute units is within 12 % of the ideal.  Shares are merged by combine_kernel.
        // Up to four rounds per die; a round halves every item longer than 0.7 of the ideal load of a
        // compute unit (so 16 shares per row tile at most).
        size_t n_live = 0;
        for (auto &v : per_die) n_live += v.size();
        std::vector<int32_t> parts_of(n_parents, 1);
        int32_t n_split_parts = 0;          // shares that need a slot in the partial-result buffer
        const auto by_cost = [](const Item &x, const Item &y) { return x.cost > y.cost; };
        if (ctx->partial && direct_kernel && n_live < (size_t)(decode_plan ? 1 : 6) * ctx->n_cus) {
            const int bins = std::max(1, ctx->n_cus / kXcds) * (tile == 128 ? 2 : 1);
            std::vector<double> heap;
            for (int d = 0; d < kXcds; ++d) {
                auto &v = per_die[d];
                for (int round = 0; round < 4 && !v.empty(); ++round) {
                    std::stable_sort(v.begin(), v.end(), by_cost);
                    // longest-first list schedule over `bins` compute units (min-heap of their loads)
                    heap.assign(bins, 0.0);
                    double total = 0;
                    for (const Item &it : v) {
                        std::pop_heap(heap.begin(), heap.end(), std::greater<double>());
                        heap.back() += it.cost;
                        std::push_heap(heap.begin(), heap.end(), std::greater<double>());
                        total += it.cost;
                    }
                    const double makespan = *std::max_element(heap.begin(), heap.end());
                    const double ideal = total / bins;
                    if (makespan <= 1.12 * ideal + 1.0) break;   // (cutting further was measured to cost more than it gains)
                    const size_t n_before = v.size();
                    bool cut_any = false;
                    for (size_t k = 0; k < n_before && v[k].cost > 0.7 * ideal; ++k) {
                        Item &it = v[k];
                        const int len = it.w.key_end - it.w.key_begin;
                        const int extra = parts_of[it.parent] == 1 ? 2 : 1;   // slots a cut of this item adds
                        if (len < 2 * kAttnMinPartKeys || parts_of[it.parent] >= kAttnMaxPartsPerTile ||
                            n_split_parts + extra > kAttnMaxParts) continue;
                        Item hi_half = it;
                        const int tiles64 = (len + 63) / 64;
                        const int mid = it.w.key_begin + (tiles64 / 2) * 64;
                        it.w.key_end = mid;
                        hi_half.w.key_begin = mid;
                        it.cost = item_cost(it.w.n_rows, mid - it.w.key_begin);
                        hi_half.cost = item_cost(hi_half.w.n_rows, hi_half.w.key_end - mid);
                        n_split_parts += extra;
                        parts_of[it.parent] += 1;
                        v.push_back(hi_half);          // (invalidates `it`)
                        cut_any = true;
                    }
                    if (!cut_any) break;
                }
                std::stable_sort(v.begin(), v.end(), by_cost);
            }
        }
        // number the shares of split row tiles consecutively and list the tiles for the merge
        CombineItem *combine = (CombineItem *)(ctx->h_meta + ctx->off_combine);
        int32_t n_combine = 0;
        {
            std::vector<int32_t> first_part(n_parents, -1), next_part(n_parents, 0);
            int32_t at = 0;
            for (auto &v : per_die)
                for (Item &it : v) {
                    if (parts_of[it.parent] == 1) continue;
                    if (first_part[it.parent] < 0) {
                        first_part[it.parent] = at;
                        at += parts_of[it.parent];
                        combine[n_combine++] = CombineItem{it.w.seq, it.w.kv_head, it.w.row0, it.w.n_rows,
                                                           first_part[it.parent], parts_of[it.parent], {0, 0}};
                    }
                    it.w.part = first_part[it.parent] + next_part[it.parent]++;
                }
            if (at != n_split_parts || at > kAttnMaxParts) return fail(ctx, CA_ERR_OUT_OF_RANGE, "ca_rope_rebase: internal: %d shares numbered, %d planned", at, n_split_parts);
        }
        ctx->n_combine = n_combine;
        ctx->n_split_parts = n_split_parts;

        size_t longest = 0;
        for (auto &v : per_die) longest = std::max(longest, v.size());
        const size_t n_items = longest * kXcds;
        if (n_items > ctx->items_capacity) return fail(ctx, CA_ERR_OUT_OF_RANGE, "ca_rope_rebase: %zu work items exceed capacity %zu", n_items, ctx->items_capacity);
        WorkItem *items = (WorkItem *)(ctx->h_meta + ctx->off_items);
        for (size_t s = 0; s < longest; ++s)
            for (int d = 0; d < kXcds; ++d)
                items[s * kXcds + d] = s < per_die[d].size() ? per_die[d][s].w : WorkItem{-1, 0, 0, 0, 0, 0, -1, 0};
        ctx->n_items = (int32_t)n_items;
    }

    // ---- order against everything still using the previous plan, then upload + per-token kernel --
    st = ca_join(ctx, stream_);
    if (st != CA_OK) return st;
    const size_t up = ctx->off_items + (size_t)ctx->n_items * sizeof(WorkItem);
    CA_HIP(ctx, hipMemcpyAsync(ctx->d_meta, ctx->h_meta, up, hipMemcpyHostToDevice, stream));
    CA_HIP(ctx, hipEventRecord(ctx->ev_meta_copied, stream));
    ctx->meta_in_flight = true;

    RebaseArgs ra{};
    ra.n_seqs = B;
    ra.max_pages = cols;
    ra.block_table = (const int32_t *)(ctx->d_meta + ctx->off_table);
    ra.n_keep = (const int32_t *)(ctx->d_meta + ctx->off_n_keep);
    ra.cu_q = (const int32_t *)(ctx->d_meta + ctx->off_cu_q);
    ra.cu_k = (const int32_t *)(ctx->d_meta + ctx->off_cu_k);
    ra.q_pos = (int32_t *)(ctx->d_meta + ctx->off_q_pos);
    ra.q_seq = (int32_t *)(ctx->d_meta + ctx->off_q_seq);
    ra.slot_map = (int32_t *)(ctx->d_meta + ctx->off_slot_map);
    ra.total_q = (int32_t)ctx->total_q;
    ra.total_k = (int32_t)ctx->total_k;
    CA_HIP(ctx, launch_rebase(ra, stream));

    // internal streams start work of this plan only after the metadata exists
    CA_HIP(ctx, hipEventRecord(ctx->ev_plan, stream));
    CA_HIP(ctx, hipStreamWaitEvent(ctx->s_copy, ctx->ev_plan, 0));
    CA_HIP(ctx, hipStreamWaitEvent(ctx->s_unpack, ctx->ev_plan, 0));
    CA_HIP(ctx, hipStreamWaitEvent(ctx->s_save, ctx->ev_plan, 0));
    std::fill(ctx->loaded.begin(), ctx->loaded.end(), 0);
    ctx->has_plan = true;
    return CA_OK;
}

ca_status ca_rebase_read(ca_ctx *ctx, int32_t which, int32_t *out, int64_t capacity, int64_t *count) {
    if (!ctx || !out || !count || capacity < 0) return CA_ERR_INVALID_ARG;
    if (!ctx->has_plan) return fail(ctx, CA_ERR_NOT_READY, "ca_rebase_read: no plan (call ca_rope_rebase first)");
    size_t off;
    int64_t n;
    switch (which) {
        case 0: off = ctx->off_n_keep; n = ctx->n_seqs; break;
        case 1: off = ctx->off_cu_q; n = ctx->n_seqs + 1; break;
        case 2: off = ctx->off_cu_k; n = ctx->n_seqs + 1; break;
        case 3: off = ctx->off_q_pos; n = ctx->total_q; break;
        case 4: off = ctx->off_q_seq; n = ctx->total_q; break;
        case 5: off = ctx->off_slot_map; n = ctx->total_k; break;
        case 6: off = ctx->off_items; n = (int64_t)ctx->n_items * 8; break;
        default: return fail(ctx, CA_ERR_INVALID_ARG, "ca_rebase_read: which = %d", which);
    }
    if (n > capacity) return fail(ctx, CA_ERR_OUT_OF_RANGE, "ca_rebase_read: need %lld elements, capacity %lld", (long long)n, (long long)capacity);
    CA_HIP(ctx, hipSetDevice(ctx->cfg.device));
    CA_HIP(ctx, hipDeviceSynchronize());
    CA_HIP(ctx, hipMemcpy(out, ctx->d_meta + off, (size_t)n * 4, hipMemcpyDeviceToHost));
    *count = n;
    return CA_OK;
}

// ----------------------------------------------------------------------------------------------
// Section 3.2: movement between the contiguous tier and the paged pool
// ----------------------------------------------------------------------------------------------
namespace {

struct Segment {  // one conversation's share of a move
    uint8_t *k, *v;
    int64_t contig_tok0;
    int32_t ctx_tok0, count, seq;
};

// narrow_workgroups > 0: launch about that many workgroups at most (each then walks several pages)
ca_status run_move(ca_ctx *ctx, bool to_pool, const std::vector<Segment> &segs, void *k_pool, void *v_pool,
                   hipStream_t stream, int narrow_workgroups = 0) {
    const ca_config &c = ctx->cfg;
    MoveShape shape{};
    shape.block_table = (const int32_t *)(ctx->d_meta + ctx->off_table);
    shape.max_pages = ctx->max_pages;
    shape.n_kv_heads = c.n_kv_heads;
    shape.vecs_per_row = c.head_dim * 2 / 16;
    // one 256-lane pass of kMoveUnroll x 16 bytes per lane covers 16 tokens of this many heads
    shape.heads_per_wg = std::max(1, std::min(c.n_kv_heads, kMoveUnroll * 256 / (16 * shape.vecs_per_row)));
    for (size_t at = 0; at < segs.size(); at += kMaxSeqsPerLaunch) {
        MoveArgs args;
        std::memset(&args, 0, sizeof args);
        const int n = (int)std::min<size_t>(kMaxSeqsPerLaunch, segs.size() - at);
        int max_touched = 0;
        for (int i = 0; i < n; ++i) {
            const Segment &s = segs[at + i];
            args.contig_k[i] = s.k;
            args.contig_v[i] = s.v;
            args.contig_tok0[i] = s.contig_tok0;
            args.ctx_tok0[i] = s.ctx_tok0;
            args.count[i] = s.count;
            args.seq[i] = s.seq;
            if (s.count > 0)
                max_touched = std::max(max_touched, (s.ctx_tok0 + s.count - 1) / kPageSize - s.ctx_tok0 / kPageSize + 1);
        }
        shape.n_in_launch = n;
        shape.max_pages_touched = max_touched;
        if (narrow_workgroups > 0) {
            const int slices = (c.n_kv_heads + shape.heads_per_wg - 1) / shape.heads_per_wg;
            shape.max_grid_y = std::max(1, narrow_workgroups / (2 * slices * n));
        }
        CA_HIP(ctx, launch_move(to_pool, args, shape, (uint8_t *)k_pool, (uint8_t *)v_pool, stream));
    }
    return CA_OK;
}

ca_status check_pools(ca_ctx *ctx, const char *who, const void *k_pool, const void *v_pool) {
    if (!k_pool || !v_pool) return fail(ctx, CA_ERR_INVALID_ARG, "%s: pool pointer is NULL", who);
    const size_t bytes = (size_t)ctx->num_pages * ctx->cfg.page_size * (size_t)row_bytes(ctx->cfg);
    if (!device_range_ok(k_pool, bytes) || !device_range_ok(v_pool, bytes))
        return fail(ctx, CA_ERR_INVALID_ARG, "%s: a pool is not device memory holding num_pages=%d pages (%zu bytes)", who,
                    ctx->num_pages, bytes);
    return CA_OK;
}

ca_status check_layer_plan(ca_ctx *ctx, const char *who, int32_t layer) {
    if (!ctx->has_plan) return fail(ctx, CA_ERR_NOT_READY, "%s: no plan (call ca_rope_rebase first)", who);
    if (layer < 0 || layer >= ctx->cfg.n_layers)
        return fail(ctx, CA_ERR_OUT_OF_RANGE, "%s: layer %d outside [0, %d)", who, layer, ctx->cfg.n_layers);
    return CA_OK;
}

}  // namespace

ca_status ca_kv_load_layer(ca_ctx *ctx, int32_t layer, const void *const *src_k, const void *const *src_v,
                           void *k_pool, void *v_pool) {
    if (!ctx) return CA_ERR_INVALID_ARG;
    ca_status st = check_layer_plan(ctx, "ca_kv_load_layer", layer);
    if (st != CA_OK) return st;
    if (!src_k || !src_v) return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_load_layer: source pointer array is NULL");
    if (ctx->loaded[layer]) return fail(ctx, CA_ERR_NOT_READY, "ca_kv_load_layer: layer %d already loaded under this plan", layer);
    const ca_config &c = ctx->cfg;
    CA_HIP(ctx, hipSetDevice(c.device));
    st = check_pools(ctx, "ca_kv_load_layer", k_pool, v_pool);
    if (st != CA_OK) return st;

    const int B = ctx->n_seqs;
    const int64_t rb = row_bytes(c);
    bool any_host = false, any_unknown = false;
    for (int i = 0; i < B; ++i) {
        if (ctx->n_keep[i] == 0) continue;
        if (!src_k[i] || !src_v[i]) return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_load_layer: source of conversation %d is NULL", i);
        const MemKind kk = mem_kind(src_k[i]), kv = mem_kind(src_v[i]);
        if (kk == MemKind::kUnknown || kv == MemKind::kUnknown) any_unknown = true;
        if (kk == MemKind::kPinnedHost || kv == MemKind::kPinnedHost) any_host = true;
        if (kk == MemKind::kDevice && !device_range_ok(src_k[i], (size_t)ctx->hist_len[i] * rb))
            return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_load_layer: K source of conversation %d is smaller than hist_len tokens", i);
        if (kv == MemKind::kDevice && !device_range_ok(src_v[i], (size_t)ctx->hist_len[i] * rb))
            return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_load_layer: V source of conversation %d is smaller than hist_len tokens", i);
    }
    if (any_unknown)
        return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_load_layer: a source is neither pinned host nor device memory");
    const bool staged = c.load_mode == 1 || (c.load_mode == 0 && any_host);

    std::vector<Segment> segs;
    segs.reserve(B);
    if (staged) {
        const int slot = (int)(ctx->load_count % c.pipeline_depth);
        uint8_t *sk = ctx->load_slots + (size_t)slot * ctx->slot_bytes;
        uint8_t *sv = sk + ctx->half_slot_bytes;
        // The K half is copied on the copy stream and the V half on the unpack stream, ahead of the kernel that needs
        // both: two copy queues keep the host link busier than one (each fills the gaps between the other's
        // per-conversation copies), and a stream of its own for the second queue would be one more than the hardware
        // queues a process has, which makes unrelated streams wait for each other.
        // the slot is free again once the unpack that last read it has finished (the unpack stream is behind it anyway)
        if (ctx->slot_used[slot]) CA_HIP(ctx, hipStreamWaitEvent(ctx->s_copy, ctx->ev_slot_free[slot], 0));
        int iv_copy;
        CA_HIP(ctx, prof_begin(ctx, kProfCopyIn, ctx->s_copy, &iv_copy));
        for (int i = 0; i < B; ++i) {
            const int64_t n = ctx->n_keep[i];
            if (n == 0) continue;
            // the kept ranges land back to back in the slot: truncation and discarding are source offsets
            size_t dst_off = (size_t)ctx->cu_n[i] * rb;
            for (int r = ctx->keep_rng_at[i]; r < ctx->keep_rng_at[i + 1]; ++r) {
                const size_t src_off = (size_t)ctx->keep_rng[r].first * rb;
                const size_t bytes = (size_t)(ctx->keep_rng[r].second - ctx->keep_rng[r].first) * rb;
                CA_HIP(ctx, hipMemcpyAsync(sk + dst_off, (const uint8_t *)src_k[i] + src_off, bytes, hipMemcpyDefault, ctx->s_copy));
                CA_HIP(ctx, hipMemcpyAsync(sv + dst_off, (const uint8_t *)src_v[i] + src_off, bytes, hipMemcpyDefault, ctx->s_unpack));
                dst_off += bytes;
            }
            segs.push_back({sk, sv, ctx->cu_n[i], 0, (int32_t)n, i});
        }
        if (iv_copy >= 0) {
            // a timed copy-in ends when both halves have landed (only then do the two queues meet once per layer)
            CA_HIP(ctx, hipEventRecord(ctx->ev_slot_copied2[slot], ctx->s_unpack));
            CA_HIP(ctx, hipStreamWaitEvent(ctx->s_copy, ctx->ev_slot_copied2[slot], 0));
        }
        CA_HIP(ctx, prof_end(ctx, iv_copy, ctx->s_copy));
        CA_HIP(ctx, hipEventRecord(ctx->ev_slot_copied[slot], ctx->s_copy));
        CA_HIP(ctx, hipStreamWaitEvent(ctx->s_unpack, ctx->ev_slot_copied[slot], 0));
        int iv_unpack;
        CA_HIP(ctx, prof_begin(ctx, kProfUnpack, ctx->s_unpack, &iv_unpack));
        st = run_move(ctx, true, segs, k_pool, v_pool, ctx->s_unpack);
        if (st != CA_OK) return st;
        CA_HIP(ctx, prof_end(ctx, iv_unpack, ctx->s_unpack));
        CA_HIP(ctx, hipEventRecord(ctx->ev_slot_free[slot], ctx->s_unpack));
        ctx->slot_used[slot] = 1;
        ctx->load_count++;
    } else {
        for (int i = 0; i < B; ++i) {
            const int64_t n = ctx->n_keep[i];
            if (n == 0) continue;
            int32_t at = 0;      // context token the range starts at
            for (int r = ctx->keep_rng_at[i]; r < ctx->keep_rng_at[i + 1]; ++r) {
                const int32_t len = ctx->keep_rng[r].second - ctx->keep_rng[r].first;
                segs.push_back({(uint8_t *)src_k[i], (uint8_t *)src_v[i], ctx->keep_rng[r].first, at, len, i});
                at += len;
            }
        }
        int iv_unpack;
        CA_HIP(ctx, prof_begin(ctx, kProfUnpack, ctx->s_unpack, &iv_unpack));
        st = run_move(ctx, true, segs, k_pool, v_pool, ctx->s_unpack);
        if (st != CA_OK) return st;
        CA_HIP(ctx, prof_end(ctx, iv_unpack, ctx->s_unpack));
    }
    CA_HIP(ctx, hipEventRecord(ctx->ev_ready[layer], ctx->s_unpack));
    ctx->loaded[layer] = 1;
    return CA_OK;
}

ca_status ca_kv_append_layer(ca_ctx *ctx, int32_t layer, const void *new_k, const void *new_v, void *k_pool,
                             void *v_pool, void *stream) {
    if (!ctx) return CA_ERR_INVALID_ARG;
    ca_status st = check_layer_plan(ctx, "ca_kv_append_layer", layer);
    if (st != CA_OK) return st;
    const ca_config &c = ctx->cfg;
    CA_HIP(ctx, hipSetDevice(c.device));
    st = check_pools(ctx, "ca_kv_append_layer", k_pool, v_pool);
    if (st != CA_OK) return st;
    const size_t bytes = (size_t)ctx->total_q * (size_t)row_bytes(c);
    if (!device_range_ok(new_k, bytes) || !device_range_ok(new_v, bytes))
        return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_append_layer: new_k/new_v must be device memory of %zu bytes", bytes);
    std::vector<Segment> segs;
    for (int i = 0; i < ctx->n_seqs; ++i)
        segs.push_back({(uint8_t *)new_k, (uint8_t *)new_v, ctx->cu_q[i], ctx->n_keep[i], ctx->new_len[i], i});
    int iv;
    CA_HIP(ctx, prof_begin(ctx, kProfAppend, (hipStream_t)stream, &iv));
    st = run_move(ctx, true, segs, k_pool, v_pool, (hipStream_t)stream);
    if (st != CA_OK) return st;
    CA_HIP(ctx, prof_end(ctx, iv, (hipStream_t)stream));
    return CA_OK;
}

ca_status ca_kv_save_layer(ca_ctx *ctx, int32_t layer, const int32_t *tok_begin, const int32_t *tok_end,
                           const void *k_pool, const void *v_pool, void *const *dst_k, void *const *dst_v,
                           const int64_t *dst_tok_offset, void *after_stream) {
    if (!ctx) return CA_ERR_INVALID_ARG;
    ca_status st = check_layer_plan(ctx, "ca_kv_save_layer", layer);
    if (st != CA_OK) return st;
    if (!dst_k || !dst_v) return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_save_layer: destination pointer array is NULL");
    if ((tok_begin == nullptr) != (tok_end == nullptr))
        return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_save_layer: tok_begin and tok_end must both be given or both NULL");
    const ca_config &c = ctx->cfg;
    CA_HIP(ctx, hipSetDevice(c.device));
    st = check_pools(ctx, "ca_kv_save_layer", k_pool, v_pool);
    if (st != CA_OK) return st;

    const int B = ctx->n_seqs;
    const int64_t rb = row_bytes(c);
    struct Range { int32_t b, e; int64_t off; };
    std::vector<Range> r(B);
    bool any_host = false;
    int64_t total = 0;
    for (int i = 0; i < B; ++i) {
        const int32_t ctx_len = ctx->n_keep[i] + ctx->new_len[i];
        r[i].b = tok_begin ? tok_begin[i] : ctx->n_keep[i];
        r[i].e = tok_end ? tok_end[i] : ctx_len;
        r[i].off = dst_tok_offset ? dst_tok_offset[i] : ctx->hist_len[i];
        if (r[i].b < 0 || r[i].e < r[i].b || r[i].e > ctx_len)
            return fail(ctx, CA_ERR_OUT_OF_RANGE, "ca_kv_save_layer: conversation %d: token range [%d, %d) outside the context [0, %d)", i,
                        r[i].b, r[i].e, ctx_len);
        if (r[i].off < 0) return fail(ctx, CA_ERR_OUT_OF_RANGE, "ca_kv_save_layer: conversation %d: negative destination offset", i);
        if (r[i].e == r[i].b) continue;
        if (!dst_k[i] || !dst_v[i]) return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_save_layer: destination of conversation %d is NULL", i);
        const MemKind kk = mem_kind(dst_k[i]), kv = mem_kind(dst_v[i]);
        if (kk == MemKind::kUnknown || kv == MemKind::kUnknown)
            return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_save_layer: destination of conversation %d is neither pinned host nor device memory", i);
        if (kk == MemKind::kPinnedHost || kv == MemKind::kPinnedHost) any_host = true;
        const size_t need = (size_t)(r[i].off + (r[i].e - r[i].b)) * rb;
        if ((kk == MemKind::kDevice && !device_range_ok(dst_k[i], need)) || (kv == MemKind::kDevice && !device_range_ok(dst_v[i], need)))
            return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_save_layer: destination of conversation %d is smaller than offset + count tokens", i);
        total += r[i].e - r[i].b;
    }
    if (total > c.max_batch_kv_tokens) return fail(ctx, CA_ERR_OUT_OF_RANGE, "ca_kv_save_layer: %lld tokens exceed a staging slot", (long long)total);
    const bool staged = any_host ? !host_save_in_place(ctx, total) : c.save_mode == 1;

    // saving starts after the producer of this layer's K/V: the work queued on `after_stream`, and the load of
    // this layer if one was issued (its unpack runs on an internal stream and may still be writing the pages a
    // range of kept-history tokens reads)
    CA_HIP(ctx, hipEventRecord(ctx->ev_after, (hipStream_t)after_stream));
    CA_HIP(ctx, hipStreamWaitEvent(ctx->s_save, ctx->ev_after, 0));
    if (ctx->loaded[layer]) CA_HIP(ctx, hipStreamWaitEvent(ctx->s_save, ctx->ev_ready[layer], 0));

    std::vector<Segment> segs;
    segs.reserve(B);
    if (staged) {
        // pack and copy-out run on the one save stream, so a slot is never overwritten while it is
        // still being copied; several slots only let the caller queue saves without bound
        const int slot = (int)(ctx->save_count % c.pipeline_depth);
        uint8_t *sk = ctx->save_slots + (size_t)slot * ctx->slot_bytes;
        uint8_t *sv = sk + ctx->half_slot_bytes;
        int64_t at = 0;
        std::vector<int64_t> slot_tok0(B, 0);
        for (int i = 0; i < B; ++i) {
            const int32_t cnt = r[i].e - r[i].b;
            if (cnt == 0) continue;
            slot_tok0[i] = at;
            segs.push_back({sk, sv, at, r[i].b, cnt, i});
            at += cnt;
        }
        int iv_pack, iv_out;
        CA_HIP(ctx, prof_begin(ctx, kProfPack, ctx->s_save, &iv_pack));
        st = run_move(ctx, false, segs, (void *)k_pool, (void *)v_pool, ctx->s_save);
        if (st != CA_OK) return st;
        CA_HIP(ctx, prof_end(ctx, iv_pack, ctx->s_save));
        CA_HIP(ctx, prof_begin(ctx, kProfCopyOut, ctx->s_save, &iv_out));
        for (int i = 0; i < B; ++i) {
            const int32_t cnt = r[i].e - r[i].b;
            if (cnt == 0) continue;
            const size_t bytes = (size_t)cnt * rb, src_off = (size_t)slot_tok0[i] * rb, dst_off = (size_t)r[i].off * rb;
            CA_HIP(ctx, hipMemcpyAsync((uint8_t *)dst_k[i] + dst_off, sk + src_off, bytes, hipMemcpyDefault, ctx->s_save));
            CA_HIP(ctx, hipMemcpyAsync((uint8_t *)dst_v[i] + dst_off, sv + src_off, bytes, hipMemcpyDefault, ctx->s_save));
        }
        CA_HIP(ctx, prof_end(ctx, iv_out, ctx->s_save));
        ctx->save_count++;
    } else {
        for (int i = 0; i < B; ++i) {
            const int32_t cnt = r[i].e - r[i].b;
            if (cnt == 0) continue;
            segs.push_back({(uint8_t *)dst_k[i], (uint8_t *)dst_v[i], r[i].off, r[i].b, cnt, i});
        }
        int iv_pack;
        CA_HIP(ctx, prof_begin(ctx, kProfPack, ctx->s_save, &iv_pack));
        // stores that cross the host link are bound by the link: a few workgroups saturate it, and a grid that filled the
        // GPU with waiting wavefronts would take the compute units from the attention kernel running beside it
        st = run_move(ctx, false, segs, (void *)k_pool, (void *)v_pool, ctx->s_save, any_host ? kHostStoreWorkgroups : 0);
        if (st != CA_OK) return st;
        CA_HIP(ctx, prof_end(ctx, iv_pack, ctx->s_save));
    }
    return CA_OK;
}

// Appending and saving the new turn in one call: the saved bytes ARE the appended bytes (keys without positions,
// Section 3.4), so the pool need not be read back.  Device destinations (and pinned ones under save_mode 2): one kernel
// reads new_k/new_v once and stores every vector twice (pool and tier).  Pinned destinations by default: append kernel,
// then the pack kernel writes the tier in place from the save stream.  Pinned destinations with staged saving: the
// copy-out on the save stream reads new_k/new_v directly; no pack kernel, no staging slot.
ca_status ca_kv_append_save_layer(ca_ctx *ctx, int32_t layer, const void *new_k, const void *new_v, void *k_pool,
                                  void *v_pool, void *const *dst_k, void *const *dst_v, void *stream_) {
    if (!ctx) return CA_ERR_INVALID_ARG;
    ca_status st = check_layer_plan(ctx, "ca_kv_append_save_layer", layer);
    if (st != CA_OK) return st;
    if (!dst_k || !dst_v) return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_append_save_layer: destination pointer array is NULL");
    const ca_config &c = ctx->cfg;
    CA_HIP(ctx, hipSetDevice(c.device));
    st = check_pools(ctx, "ca_kv_append_save_layer", k_pool, v_pool);
    if (st != CA_OK) return st;
    const int64_t rb = row_bytes(c);
    const size_t bytes = (size_t)ctx->total_q * (size_t)rb;
    if (!device_range_ok(new_k, bytes) || !device_range_ok(new_v, bytes))
        return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_append_save_layer: new_k/new_v must be device memory of %zu bytes", bytes);
    const int B = ctx->n_seqs;
    bool any_host = false;
    for (int i = 0; i < B; ++i) {
        if (!dst_k[i] || !dst_v[i]) return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_append_save_layer: destination of conversation %d is NULL", i);
        const MemKind kk = mem_kind(dst_k[i]), kv = mem_kind(dst_v[i]);
        if (kk == MemKind::kUnknown || kv == MemKind::kUnknown)
            return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_append_save_layer: destination of conversation %d is neither pinned host nor device memory", i);
        if (kk == MemKind::kPinnedHost || kv == MemKind::kPinnedHost) any_host = true;
        const size_t need = (size_t)(ctx->hist_len[i] + ctx->new_len[i]) * rb;
        if ((kk == MemKind::kDevice && !device_range_ok(dst_k[i], need)) || (kv == MemKind::kDevice && !device_range_ok(dst_v[i], need)))
            return fail(ctx, CA_ERR_INVALID_ARG, "ca_kv_append_save_layer: destination of conversation %d is smaller than hist_len + new_len tokens", i);
    }
    const bool staged = any_host ? !host_save_in_place(ctx, ctx->total_q) : c.save_mode == 1;
    hipStream_t stream = (hipStream_t)stream_;
    if (!staged && any_host && c.save_mode == 0) {
        // a pinned tier: the append kernel on the caller's stream, then the pack kernel on the save stream writes the
        // new tokens to the tier in place (the caller's stream must not wait for stores that cross the host link)
        std::vector<Segment> segs;
        for (int i = 0; i < B; ++i)
            segs.push_back({(uint8_t *)new_k, (uint8_t *)new_v, ctx->cu_q[i], ctx->n_keep[i], ctx->new_len[i], i});
        int iv;
        CA_HIP(ctx, prof_begin(ctx, kProfAppend, stream, &iv));
        st = run_move(ctx, true, segs, k_pool, v_pool, stream);
        if (st != CA_OK) return st;
        CA_HIP(ctx, prof_end(ctx, iv, stream));
        CA_HIP(ctx, hipEventRecord(ctx->ev_after, stream));
        CA_HIP(ctx, hipStreamWaitEvent(ctx->s_save, ctx->ev_after, 0));
        if (ctx->loaded[layer]) CA_HIP(ctx, hipStreamWaitEvent(ctx->s_save, ctx->ev_ready[layer], 0));
        segs.clear();
        for (int i = 0; i < B; ++i)
            if (ctx->new_len[i] > 0)
                segs.push_back({(uint8_t *)dst_k[i], (uint8_t *)dst_v[i], ctx->hist_len[i], ctx->n_keep[i], ctx->new_len[i], i});
        int iv_pack;
        CA_HIP(ctx, prof_begin(ctx, kProfPack, ctx->s_save, &iv_pack));
        st = run_move(ctx, false, segs, k_pool, v_pool, ctx->s_save, kHostStoreWorkgroups);
        if (st != CA_OK) return st;
        CA_HIP(ctx, prof_end(ctx, iv_pack, ctx->s_save));
        return CA_OK;
    }
    if (staged) {
        // append on the caller's stream; the copy-out follows it on the save stream, straight from new_k / new_v
        std::vector<Segment> segs;
        for (int i = 0; i < B; ++i)
            segs.push_back({(uint8_t *)new_k, (uint8_t *)new_v, ctx->cu_q[i], ctx->n_keep[i], ctx->new_len[i], i});
        int iv;
        CA_HIP(ctx, prof_begin(ctx, kProfAppend, stream, &iv));
        st = run_move(ctx, true, segs, k_pool, v_pool, stream);
        if (st != CA_OK) return st;
        CA_HIP(ctx, prof_end(ctx, iv, stream));
        CA_HIP(ctx, hipEventRecord(ctx->ev_after, stream));
        CA_HIP(ctx, hipStreamWaitEvent(ctx->s_save, ctx->ev_after, 0));
        int iv_out;
        CA_HIP(ctx, prof_begin(ctx, kProfCopyOut, ctx->s_save, &iv_out));
        for (int i = 0; i < B; ++i) {
            const size_t n = (size_t)ctx->new_len[i] * rb, src_off = (size_t)ctx->cu_q[i] * rb, dst_off = (size_t)ctx->hist_len[i] * rb;
            CA_HIP(ctx, hipMemcpyAsync((uint8_t *)dst_k[i] + dst_off, (const uint8_t *)new_k + src_off, n, hipMemcpyDefault, ctx->s_save));
            CA_HIP(ctx, hipMemcpyAsync((uint8_t *)dst_v[i] + dst_off, (const uint8_t *)new_v + src_off, n, hipMemcpyDefault, ctx->s_save));
        }
        CA_HIP(ctx, prof_end(ctx, iv_out, ctx->s_save));
        return CA_OK;
    }
    // one pass: every vector of the new turn goes to its page and to its row of the tier
    MoveShape shape{};
    shape.block_table = (const int32_t *)(ctx->d_meta + ctx->off_table);
    shape.max_pages = ctx->max_pages;
    shape.n_kv_heads = c.n_kv_heads;
    shape.vecs_per_row = c.head_dim * 2 / 16;
    shape.heads_per_wg = std::max(1, std::min(c.n_kv_heads, kMoveUnroll * 256 / (16 * shape.vecs_per_row)));
    int iv;
    CA_HIP(ctx, prof_begin(ctx, kProfAppend, stream, &iv));
    for (int at = 0; at < B; at += kMaxSeqsPerLaunch) {
        MoveArgs args;
        MoveArgs2 second;
        std::memset(&args, 0, sizeof args);
        std::memset(&second, 0, sizeof second);
        const int n = std::min(kMaxSeqsPerLaunch, B - at);
        int max_touched = 0;
        for (int i = 0; i < n; ++i) {
            const int q = at + i;
            args.contig_k[i] = (uint8_t *)new_k;
            args.contig_v[i] = (uint8_t *)new_v;
            args.contig_tok0[i] = ctx->cu_q[q];
            args.ctx_tok0[i] = ctx->n_keep[q];
            args.count[i] = ctx->new_len[q];
            args.seq[i] = q;
            second.dst2_k[i] = (uint8_t *)dst_k[q];
            second.dst2_v[i] = (uint8_t *)dst_v[q];
            second.dst2_tok0[i] = ctx->hist_len[q];       // new token j is saved behind the history, at token hist_len + j
            max_touched = std::max(max_touched, (ctx->n_keep[q] + ctx->new_len[q] - 1) / kPageSize - ctx->n_keep[q] / kPageSize + 1);
        }
        shape.n_in_launch = n;
        shape.max_pages_touched = max_touched;
        CA_HIP(ctx, launch_move_dual(args, second, shape, (uint8_t *)k_pool, (uint8_t *)v_pool, stream));
    }
    CA_HIP(ctx, prof_end(ctx, iv, stream));
    return CA_OK;
}

// ----------------------------------------------------------------------------------------------
// Sections 2.1 / 3.1 / 3.4: attention of the new tokens
// ----------------------------------------------------------------------------------------------
// partial: where the shares of split row tiles go (the context's buffer, or the static scratch array);
// timed: bracket the launch with profiling events when profiling is on (creating an event may allocate)
static ca_status attn_impl(ca_ctx *ctx, int32_t layer, const void *q, const void *k_pool, const void *v_pool, void *out,
                           float softmax_scale, void *stream_, float *partial, bool timed) {
    ca_status st = check_layer_plan(ctx, "ca_cached_prefill_attn", layer);
    if (st != CA_OK) return st;
    const ca_config &c = ctx->cfg;
    CA_HIP(ctx, hipSetDevice(c.device));
    st = check_pools(ctx, "ca_cached_prefill_attn", k_pool, v_pool);
    if (st != CA_OK) return st;
    if (!(softmax_scale > 0.f) || !std::isfinite(softmax_scale))
        return fail(ctx, CA_ERR_INVALID_ARG, "ca_cached_prefill_attn: softmax_scale must be finite and > 0");
    const size_t q_bytes = (size_t)ctx->total_q * c.n_q_heads * c.head_dim * 2;
    if (!device_range_ok(q, q_bytes) || !device_range_ok(out, q_bytes))
        return fail(ctx, CA_ERR_INVALID_ARG, "ca_cached_prefill_attn: q/out must be device memory of %zu bytes", q_bytes);
    hipStream_t stream = (hipStream_t)stream_;
    if (ctx->loaded[layer]) {
        CA_HIP(ctx, hipStreamWaitEvent(stream, ctx->ev_ready[layer], 0));
    } else if (c.require_load && ctx->total_n > 0) {
        return fail(ctx, CA_ERR_NOT_READY, "ca_cached_prefill_attn: layer %d has kept history but was not loaded under this plan", layer);
    }
    AttnArgs a{};
    a.q = (const uint16_t *)q;
    a.out = (uint16_t *)out;
    a.k_pool = (const uint16_t *)k_pool;
    a.v_pool = (const uint16_t *)v_pool;
    a.block_table = (const int32_t *)(ctx->d_meta + ctx->off_table);
    a.n_keep = (const int32_t *)(ctx->d_meta + ctx->off_n_keep);
    a.cu_q = (const int32_t *)(ctx->d_meta + ctx->off_cu_q);
    a.q_pos = (const int32_t *)(ctx->d_meta + ctx->off_q_pos);
    a.q_seq = (const int32_t *)(ctx->d_meta + ctx->off_q_seq);
    a.items = (const WorkItem *)(ctx->d_meta + ctx->off_items);
    a.combine = (const CombineItem *)(ctx->d_meta + ctx->off_combine);
    a.partial = partial;
    a.k_rot = ctx->k_rot;
    a.dense_page0 = (const int32_t *)(ctx->d_meta + ctx->off_dense0);
    a.rot_src_page = (const int32_t *)(ctx->d_meta + ctx->off_rot_src);
    a.rot_pos0 = (const int32_t *)(ctx->d_meta + ctx->off_rot_pos);
    a.v_t = ctx->v_t;
    a.rot_nvalid = (const int32_t *)(ctx->d_meta + ctx->off_rot_nvalid);
    a.pipelined = ctx->pipelined ? 1 : 0;
    a.n_dense_pages = ctx->n_dense_pages;
    a.prerotate = ctx->prerotate ? 1 : 0;
    a.max_positions = c.max_positions;
    a.n_combine = ctx->n_combine;
    a.rope = ctx->rope;
    a.n_items = ctx->n_items;
    a.total_q = (int32_t)ctx->total_q;
    a.max_pages = ctx->max_pages;
    a.n_q_heads = c.n_q_heads;
    a.n_kv_heads = c.n_kv_heads;
    a.head_dim = c.head_dim;
    a.rope_style = c.rope_style;
    a.tile_rows = ctx->tile_rows;
    a.softmax_scale = softmax_scale;
    int iv = -1;
    if (timed) CA_HIP(ctx, prof_begin(ctx, kProfAttn, stream, &iv));
    // 0 picks the LDS-direct kernel whenever its page-id table holds the window
    const bool direct = direct_variant(c);
    // a decode step (one or two stacked rows per (conversation, kv head)) is a matrix-vector product: streamed
    const bool decode = direct && c.attn_variant != 2 && !ctx->prerotate && ctx->max_unit_rows >= 1 &&
                        ctx->max_unit_rows <= kAttnDecodeMaxRows;
    if (c.attn_variant == 4 && !decode) {
        (void)prof_end(ctx, iv, stream);
        return fail(ctx, CA_ERR_UNSUPPORTED, "ca_cached_prefill_attn: attn_variant 4 needs at most %d stacked rows per (conversation, kv head), the plan has %d",
                    kAttnDecodeMaxRows, ctx->max_unit_rows);
    }
    if (c.attn_variant == 1) {
        CA_HIP(ctx, launch_attn_ref(a, stream));
    } else if (decode) {
        CA_HIP(ctx, launch_attn_decode(a, ctx->max_unit_rows, stream));
    } else if (direct && ctx->pipelined) {
        CA_HIP(ctx, launch_attn_pp(a, stream));
    } else if (direct) {
        CA_HIP(ctx, launch_attn_dma(a, stream));
    } else {
        return fail(ctx, CA_ERR_UNSUPPORTED, "ca_cached_prefill_attn: attn_variant %d", c.attn_variant);
    }
    CA_HIP(ctx, prof_end(ctx, iv, stream));
    return CA_OK;
}

ca_status ca_cached_prefill_attn(ca_ctx *ctx, int32_t layer, const void *q, const void *k_pool, const void *v_pool,
                                 void *out, float softmax_scale, void *stream) {
    if (!ctx) return CA_ERR_INVALID_ARG;
    return attn_impl(ctx, layer, q, k_pool, v_pool, out, softmax_scale, stream, ctx->partial, true);
}

ca_status ca_cached_prefill_attn_static(ca_ctx *ctx, int32_t layer, const void *q, const void *k_pool, const void *v_pool,
                                        void *out, float softmax_scale, void *stream) {
    if (!ctx) return CA_ERR_INVALID_ARG;
    if (ctx->has_plan && ctx->n_split_parts > 0) {
        if (!ctx->static_partial)
            return fail(ctx, CA_ERR_UNSUPPORTED, "ca_cached_prefill_attn_static: no static scratch on device %d", ctx->cfg.device);
        const size_t need = (size_t)ctx->n_split_parts * (size_t)ctx->tile_rows * (size_t)(ctx->cfg.head_dim + 2) * sizeof(float);
        if (need > kStaticScratchBytes)
            return fail(ctx, CA_ERR_OUT_OF_RANGE, "ca_cached_prefill_attn_static: the plan's %d shares of split row tiles need %zu bytes of "
                        "partial results, the static scratch holds %zu", ctx->n_split_parts, need, kStaticScratchBytes);
    }
    return attn_impl(ctx, layer, q, k_pool, v_pool, out, softmax_scale, stream, ctx->static_partial, false);
}

// ----------------------------------------------------------------------------------------------
// timing of the library's own GPU work
// ----------------------------------------------------------------------------------------------
ca_status ca_profile_enable(ca_ctx *ctx, int32_t on) {
    if (!ctx) return CA_ERR_INVALID_ARG;
    ctx->profiling = on != 0;
    ctx->profile_mask = (on == 1 || on == 0) ? ~0u : ((uint32_t)on >> 1);
    return CA_OK;
}

ca_status ca_profile_read(ca_ctx *ctx, int32_t kind, double *total_ms, int64_t *count) {
    if (!ctx || !total_ms || !count) return CA_ERR_INVALID_ARG;
    if (kind < 0 || kind >= kProfKinds) return fail(ctx, CA_ERR_INVALID_ARG, "ca_profile_read: kind %d", kind);
    CA_HIP(ctx, hipSetDevice(ctx->cfg.device));
    CA_HIP(ctx, hipDeviceSynchronize());
    double sum = 0.0;
    int64_t n = 0;
    std::vector<ca_ctx::Interval> keep;
    for (auto &iv : ctx->intervals) {
        if (iv.kind != kind) { keep.push_back(iv); continue; }
        float ms = 0.f;
        CA_HIP(ctx, hipEventElapsedTime(&ms, iv.start, iv.stop));
        sum += ms;
        ++n;
        ctx->spare_events.push_back(iv.start);
        ctx->spare_events.push_back(iv.stop);
    }
    ctx->intervals.swap(keep);
    *total_ms = sum;
    *count = n;
    return CA_OK;
}

ca_status ca_profile_timeline(ca_ctx *ctx, int32_t *kinds, double *start_ms, double *stop_ms, int64_t capacity,
                              int64_t *count) {
    if (!ctx || !count || capacity < 0) return CA_ERR_INVALID_ARG;
    if (capacity > 0 && (!kinds || !start_ms || !stop_ms)) return fail(ctx, CA_ERR_INVALID_ARG, "ca_profile_timeline: null array");
    CA_HIP(ctx, hipSetDevice(ctx->cfg.device));
    CA_HIP(ctx, hipDeviceSynchronize());
    *count = (int64_t)ctx->intervals.size();
    const int64_t n = std::min<int64_t>(*count, capacity);
    for (int64_t i = 0; i < n; ++i) {
        const auto &iv = ctx->intervals[(size_t)i];
        float a = 0.f, b = 0.f;
        if (i > 0) CA_HIP(ctx, hipEventElapsedTime(&a, ctx->intervals[0].start, iv.start));
        CA_HIP(ctx, hipEventElapsedTime(&b, iv.start, iv.stop));
        kinds[i] = iv.kind;
        start_ms[i] = a;
        stop_ms[i] = (double)a + b;
    }
    return CA_OK;
}

}  // extern "C"
