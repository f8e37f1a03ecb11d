// Data-movement kernels of the layer-wise load / save path (Section 3.2) and the per-token
// metadata of the rebased plan (Section 3.4).  Pure integer indexing and 16-byte copies:
// results are bit-exact by construction.
//
// HBM-bound.  Per token and layer the kernels move n_kv_heads*head_dim*2 bytes of K and as many
// of V, read once and written once.  For a fixed head, 16 consecutive context tokens are one whole
// (page, head) block of the pool (4 KiB contiguous) on the paged side and 16 rows of 256 B on the
// contiguous side, so both sides move in full 256-byte segments; all heads of a page together are
// one contiguous run on either side (n_kv_heads * 4 KiB in the pool, 16 whole token rows in the
// contiguous layout).
#include "ca_internal.h"

namespace ca {

namespace {

typedef __attribute__((ext_vector_type(4))) unsigned int vec16;  // one 16-byte piece

constexpr int kMoveThreads = 256;
constexpr int kUnroll = kMoveUnroll;
constexpr int kMoveMaxGridY = 32768;

// grid: x = (slice of heads, K or V), y = page of the conversation's context (counted from the first
// page the range touches), z = conversation entry of this launch.  A workgroup moves, for one of the
// two arrays, the tokens of its page that lie inside the range for heads_per_wg heads, kUnroll loads
// of 16 bytes in flight per lane before the first store.  The page id is uniform over the workgroup.
// The order matters: x is the fastest launch dimension, so the workgroups that together cover one
// page run next to each other and both sides of the copy see long sequential runs; with few loads
// in flight per lane and keys and values in separate workgroups the kernel reaches 5.7 TB/s on a
// 337 MB load where the opposite choices (pages fastest, 4 + 4 loads per lane) gave 5.0.
// kDual (with kToPool): every vector read from the contiguous side is stored twice, into the pool and into a second
// contiguous destination (the tier): the new turn's K/V are appended and saved in one pass over them.
template <bool kToPool, bool kNT, bool kDual>
__device__ inline void move_body(const MoveArgs &a, const MoveShape &s, uint8_t *__restrict__ k_pool,
                                 uint8_t *__restrict__ v_pool, const MoveArgs2 &b) {
    static_assert(!kDual || kToPool, "the second destination goes with contiguous -> pages");
    const int e = blockIdx.z;  // entry of this launch
    const bool values = blockIdx.x & 1;
    const int ctx_begin = a.ctx_tok0[e];
    const int ctx_end = ctx_begin + a.count[e];
    // grid.y is capped below the launch limit; longer ranges take more than one trip
    for (int col = blockIdx.y; col < s.max_pages_touched; col += gridDim.y) {
        const int page_col = ctx_begin / kPageSize + col;
        const int t_first = max(ctx_begin, page_col * kPageSize);
        const int t_last = min(ctx_end, (page_col + 1) * kPageSize);   // exclusive
        if (t_first >= t_last) break;   // past the last page of this range
        const int slot0 = t_first - page_col * kPageSize;
        const int n_tok = t_last - t_first;
        const int vpr = s.vecs_per_row;
        const int H = s.n_kv_heads;
        const int h_first = (blockIdx.x >> 1) * s.heads_per_wg;
        const int h_count = min(s.heads_per_wg, H - h_first);
        const int page = s.block_table[(int64_t)a.seq[e] * s.max_pages + page_col];
        const int64_t row_vecs = (int64_t)H * vpr;  // 16-byte vectors per token on the contiguous side
        const int64_t contig_first = a.contig_tok0[e] + (t_first - ctx_begin);
        vec16 *contig = reinterpret_cast<vec16 *>(values ? a.contig_v[e] : a.contig_k[e]) + contig_first * row_vecs + (int64_t)h_first * vpr;
        vec16 *pool = reinterpret_cast<vec16 *>(values ? v_pool : k_pool) + (((int64_t)page * H + h_first) * kPageSize + slot0) * vpr;
        vec16 *second = nullptr;
        if (kDual) second = reinterpret_cast<vec16 *>(values ? b.dst2_v[e] : b.dst2_k[e]) + (b.dst2_tok0[e] + (t_first - ctx_begin)) * row_vecs + (int64_t)h_first * vpr;

        // vector id v -> (head, token, 16-byte piece), piece fastest
        const int per_head = n_tok * vpr;
        const int total = h_count * per_head;
        const int head_stride_pool = kPageSize * vpr;
        for (int v0 = threadIdx.x; v0 < total; v0 += kMoveThreads * kUnroll) {
            vec16 r[kUnroll];
            int pool_idx[kUnroll];
            int64_t contig_idx[kUnroll];
            bool live[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int v = v0 + u * kMoveThreads;
                const int hl = v / per_head;
                const int rem = v - hl * per_head;
                const int ti = rem / vpr;
                const int piece = rem - ti * vpr;
                live[u] = v < total;
                pool_idx[u] = hl * head_stride_pool + ti * vpr + piece;
                contig_idx[u] = (int64_t)ti * row_vecs + hl * vpr + piece;
                if (live[u]) {
                    const vec16 *src = kToPool ? contig + contig_idx[u] : pool + pool_idx[u];
                    r[u] = kNT ? __builtin_nontemporal_load(src) : *src;
                }
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                if (live[u]) {
                    vec16 *dst = kToPool ? pool + pool_idx[u] : contig + contig_idx[u];
                    if (kNT) __builtin_nontemporal_store(r[u], dst); else *dst = r[u];
                    if (kDual) __builtin_nontemporal_store(r[u], second + contig_idx[u]);
                }
            }
        }
    }
}

template <bool kToPool, bool kNT>
__global__ __launch_bounds__(kMoveThreads) void move_kernel(MoveArgs a, MoveShape s, uint8_t *__restrict__ k_pool,
                                                            uint8_t *__restrict__ v_pool) {
    move_body<kToPool, kNT, false>(a, s, k_pool, v_pool, MoveArgs2{});
}

__global__ __launch_bounds__(kMoveThreads) void move_dual_kernel(MoveArgs a, MoveArgs2 b, MoveShape s, uint8_t *__restrict__ k_pool,
                                                                 uint8_t *__restrict__ v_pool) {
    move_body<true, true, true>(a, s, k_pool, v_pool, b);
}

// One thread per context token: which conversation it belongs to (binary search in the prefix
// sums), where it lives in the pool, and for new tokens their rebased position.
__global__ __launch_bounds__(256) void rebase_kernel(RebaseArgs a) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.total_k) return;
    int lo = 0, hi = a.n_seqs;  // largest c with cu_k[c] <= i
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.cu_k[mid] <= i) lo = mid; else hi = mid;
    }
    const int c = lo;
    const int t = i - a.cu_k[c];
    const int page = a.block_table[(int64_t)c * a.max_pages + t / kPageSize];
    a.slot_map[i] = page * kPageSize + t % kPageSize;
    const int n = a.n_keep[c];
    if (t >= n) {
        const int j = t - n;
        a.q_pos[a.cu_q[c] + j] = t;  // new token j sits at position n + j of the truncated context
        a.q_seq[a.cu_q[c] + j] = c;
    }
}

}  // namespace

hipError_t launch_move(bool to_pool, const MoveArgs &args, const MoveShape &shape, uint8_t *k_pool,
                       uint8_t *v_pool, hipStream_t stream) {
    if (shape.n_in_launch <= 0 || shape.max_pages_touched <= 0) return hipSuccess;
    const int slices = (shape.n_kv_heads + shape.heads_per_wg - 1) / shape.heads_per_wg;
    int rows = std::min(shape.max_pages_touched, kMoveMaxGridY);
    if (shape.max_grid_y > 0) rows = std::min(rows, shape.max_grid_y);
    dim3 grid(2 * slices, rows, shape.n_in_launch);
    // nontemporal accesses: every byte is touched once (measured ~5 % faster than cached ones)
    if (to_pool)
        hipLaunchKernelGGL((move_kernel<true, true>), grid, dim3(kMoveThreads), 0, stream, args, shape, k_pool, v_pool);
    else
        hipLaunchKernelGGL((move_kernel<false, true>), grid, dim3(kMoveThreads), 0, stream, args, shape, k_pool, v_pool);
    return hipGetLastError();
}

hipError_t launch_move_dual(const MoveArgs &args, const MoveArgs2 &second, const MoveShape &shape, uint8_t *k_pool,
                            uint8_t *v_pool, hipStream_t stream) {
    if (shape.n_in_launch <= 0 || shape.max_pages_touched <= 0) return hipSuccess;
    const int slices = (shape.n_kv_heads + shape.heads_per_wg - 1) / shape.heads_per_wg;
    dim3 grid(2 * slices, std::min(shape.max_pages_touched, kMoveMaxGridY), shape.n_in_launch);
    hipLaunchKernelGGL(move_dual_kernel, grid, dim3(kMoveThreads), 0, stream, args, second, shape, k_pool, v_pool);
    return hipGetLastError();
}

hipError_t launch_rebase(const RebaseArgs &args, hipStream_t stream) {
    if (args.total_k <= 0) return hipSuccess;
    dim3 grid((args.total_k + 255) / 256);
    hipLaunchKernelGGL(rebase_kernel, grid, dim3(256), 0, stream, args);
    return hipGetLastError();
}

}  // namespace ca
