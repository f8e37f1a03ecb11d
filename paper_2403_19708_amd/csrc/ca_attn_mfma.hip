// Fused rotary-on-load + causal varlen prefill attention on the bf16 matrix cores of gfx950
// (Sections 2.1, 3.1, 3.4): the new tokens' queries attend to [kept history | new tokens] read
// from the paged pool; keys are stored without positional encoding and are rotated to their
// rebased positions on the way from HBM to LDS, so the pool is never rewritten.
//
// Work decomposition
//   One workgroup of NW wavefronts owns a tile of 32*NW stacked query rows of one (conversation,
//   kv head): row r is new token r / G under query head kv_head*G + r % G, so under GQA all G
//   heads of a group share every K/V tile that is staged.  Each wavefront owns 32 rows.
//   Keys are walked in tiles of 64, double-buffered in LDS: while tile i is multiplied, the
//   registers already hold tile i+1 (fetched one iteration earlier) and the loads of tile i+2
//   are issued, so HBM/L2 latency is covered by one whole tile of compute and there is a single
//   workgroup barrier per tile.
//
// Matrix-core formulation (v_mfma_f32_32x32x16_bf16, operands A: 32x16, B: 16x32, C: 32x32)
//   S^T = K Q^T : A = K tile rows from LDS, B = rotated Q held in registers.  In the C layout a
//   lane owns ONE query column (lane % 32) and 16 keys per 32-key block, so the softmax row
//   reductions are in-lane plus one exchange between lane l and l^32.
//   O^T += V^T P^T : A = V^T from LDS (V is transposed on its way into LDS), B = P^T, which is
//   exactly the C registers of S^T converted to bf16: no shuffle between the two products, and
//   the running rescale factor is a per-lane scalar.  The key order inside a 16-key group that
//   the C layout imposes on P^T is applied to V^T when it is written to LDS.
//
// Rotary encoding of K (Section 3.4).  Rebased positions are dense: key t of the context has
// position t.  A thread always handles the same in-tile key and the same rotary pairs, so it
// keeps their (cos, sin) in registers, initialised from the fp64-built table at position t and
// advanced from tile to tile by the fixed rotation of 64 positions (4 fp32 ops per pair, no
// table traffic in the loop; drift after 64 tiles is ~1e-5, far below the bf16 rounding of K).
//
// Softmax rescaling is lazy: the running maximum of a row is only raised (and O, l rescaled)
// when some row of the wavefront exceeds it by more than 2^8; probabilities are then bounded by
// 2^8, which bf16 and the fp32 accumulators hold without loss.
//
// Rounding: rotation in fp32 from bf16 inputs, result rounded (RNE) to bf16; scores, softmax
// statistics and both accumulators in fp32; probabilities rounded to bf16 for the second
// product; output rounded to bf16.
#include "ca_internal.h"

#include <type_traits>

namespace ca {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BN = 64;  // keys per tile

__device__ inline float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ inline uint32_t pack_bf16(float a, float b) {
    bf16x2 v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(uint32_t, v);
}

// Rotates the 8+8 elements of two 16-byte pieces `a` (dims d0..d0+7) and `b` in fp32 and rounds
// to bf16.  STYLE 0: element e of `a` pairs with element e of `b` (dims i and i + D/2), cs[e] is
// the (cos, sin) of pair d0+e.  STYLE 1: neighbours pair up inside each piece; cs[0..3] belong
// to `a`, cs[4..7] to `b`.
template <int STYLE>
__device__ inline void rotate16(uint4 &a, uint4 &b, const float2 (&cs)[8]) {
    uint32_t *pa = reinterpret_cast<uint32_t *>(&a);
    uint32_t *pb = reinterpret_cast<uint32_t *>(&b);
    if (STYLE == 0) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float a0 = bf_lo(pa[w]), a1 = bf_hi(pa[w]);
            const float b0 = bf_lo(pb[w]), b1 = bf_hi(pb[w]);
            const float2 c0 = cs[2 * w], c1 = cs[2 * w + 1];
            pa[w] = pack_bf16(a0 * c0.x - b0 * c0.y, a1 * c1.x - b1 * c1.y);
            pb[w] = pack_bf16(b0 * c0.x + a0 * c0.y, b1 * c1.x + a1 * c1.y);
        }
    } else {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float a0 = bf_lo(pa[w]), a1 = bf_hi(pa[w]);
            const float b0 = bf_lo(pb[w]), b1 = bf_hi(pb[w]);
            const float2 ca_ = cs[w], cb_ = cs[4 + w];
            pa[w] = pack_bf16(a0 * ca_.x - a1 * ca_.y, a1 * ca_.x + a0 * ca_.y);
            pb[w] = pack_bf16(b0 * cb_.x - b1 * cb_.y, b1 * cb_.x + b0 * cb_.y);
        }
    }
}

// (cos, sin) of the 8 rotary pairs that belong to pieces `piece` (dims 8*piece..) and its partner
// at +D/2, at position `pos`.
template <int D, int STYLE>
__device__ inline void load_cs(const float2 *__restrict__ rope, int pos, int piece, float2 (&cs)[8]) {
    constexpr int HALF = D / 2;
    const float2 *row = rope + (int64_t)pos * HALF;
    if (STYLE == 0) {
        const float4 *p = reinterpret_cast<const float4 *>(row + 8 * piece);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float4 v = p[w];
            cs[2 * w] = make_float2(v.x, v.y);
            cs[2 * w + 1] = make_float2(v.z, v.w);
        }
    } else {
        const float4 *p = reinterpret_cast<const float4 *>(row + 4 * piece);
        const float4 *q = reinterpret_cast<const float4 *>(row + HALF / 2 + 4 * piece);
#pragma unroll
        for (int w = 0; w < 2; ++w) {
            const float4 v = p[w], u = q[w];
            cs[2 * w] = make_float2(v.x, v.y);
            cs[2 * w + 1] = make_float2(v.z, v.w);
            cs[4 + 2 * w] = make_float2(u.x, u.y);
            cs[4 + 2 * w + 1] = make_float2(u.z, u.w);
        }
    }
}

template <int D, int STYLE, int NW>
__global__ __launch_bounds__(64 * NW, 2) void attn_mfma_kernel(AttnArgs a) {
    constexpr int NTHREADS = 64 * NW;
    constexpr int HALF = D / 2;
    constexpr int KSTEPS = D / 16;      // k-steps of the S^T product
    constexpr int PIECES = D / 16;      // 16-byte pieces in half a row
    constexpr int DBLKS = D / 32;       // 32-row blocks of O^T
    constexpr int KS_STRIDE = D + 8;    // bf16 elements; +16 bytes keeps ds_read_b128 conflict-free
    constexpr int VT_STRIDE = BN + 8;
    constexpr int K_TASKS = BN * PIECES;             // (key, piece) pairs of a K tile
    constexpr int V_TASKS = (BN / 4) * (D / 8);      // (key quad, 8-dim chunk) pairs of a V tile
    constexpr int KT = (K_TASKS + NTHREADS - 1) / NTHREADS;  // K tasks per thread
    static_assert(V_TASKS <= NTHREADS, "one V task per thread at most");
    static_assert(NTHREADS % PIECES == 0, "a thread keeps its piece across its K tasks");

    __shared__ __attribute__((aligned(16))) uint16_t Ks[2][BN * KS_STRIDE];
    __shared__ __attribute__((aligned(16))) uint16_t Vt[2][D * VT_STRIDE];

    const WorkItem item = a.items[blockIdx.x];
    if (item.seq < 0) return;

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int lq = lane & 31;
    const int half = lane >> 5;

    const int c = item.seq;
    const int g = item.kv_head;
    const int G = a.n_q_heads / a.n_kv_heads;
    const int n = a.n_keep[c];
    const int q0 = a.cu_q[c];
    const int32_t *table = a.block_table + (int64_t)c * a.max_pages;
    const int Hkv = a.n_kv_heads;

    const int row_last = item.row0 + item.n_rows - 1;          // last valid stacked row of the tile
    const int kmax = n + row_last / G + 1;                      // keys this tile can see
    const int n_tiles = (kmax + BN - 1) / BN;

    // ---- this lane's query row --------------------------------------------------------------
    const int r_raw = item.row0 + wave * 32 + lq;
    const bool row_valid = r_raw <= row_last;
    const int r = row_valid ? r_raw : row_last;
    const int j = r / G;
    const int head = g * G + (r - j * G);
    const int qpos = n + j;                                      // keys 0..qpos are visible
    // wave-uniform bounds (rows of a wave are consecutive)
    const int wr_first = min(item.row0 + wave * 32, row_last);
    const int wr_last = min(item.row0 + wave * 32 + 31, row_last);
    const bool wave_live = item.row0 + wave * 32 <= row_last;
    const int wq_min = n + wr_first / G;
    const int wq_max = n + wr_last / G;

    bf16x8 Qf[KSTEPS];
    {
        const uint16_t *qrow = a.q + ((int64_t)(q0 + j) * a.n_q_heads + head) * D;
#pragma unroll
        for (int ks = 0; ks < KSTEPS / 2; ++ks) {
            // pieces at dims 16ks + 8half (k-step ks) and the same + D/2 (k-step ks + KSTEPS/2)
            const int piece = 2 * ks + half;
            uint4 x = *reinterpret_cast<const uint4 *>(qrow + 8 * piece);
            uint4 y = *reinterpret_cast<const uint4 *>(qrow + HALF + 8 * piece);
            float2 cs[8];
            load_cs<D, STYLE>(a.rope, qpos, piece, cs);
            rotate16<STYLE>(x, y, cs);
            Qf[ks] = __builtin_bit_cast(bf16x8, x);
            Qf[ks + KSTEPS / 2] = __builtin_bit_cast(bf16x8, y);
        }
    }

    // ---- producer state: which part of every K / V tile this thread moves -----------------------
    // K task u of this thread: key kk[u] = (tid + u*NTHREADS) / PIECES, piece = tid % PIECES.
    const int k_piece = tid % PIECES;
    float2 k_step[8];          // rotation by BN positions for this thread's 8 pairs
    float2 k_cs[KT][8];        // (cos, sin) at the current tile's position of task u
    load_cs<D, STYLE>(a.rope, BN, k_piece, k_step);
#pragma unroll
    for (int u = 0; u < KT; ++u) load_cs<D, STYLE>(a.rope, (tid + u * NTHREADS) / PIECES, k_piece, k_cs[u]);
    // V task: quad of keys 4*v_kq.., dims 8*v_dc..; lanes of a wavefront walk the key quads so that the
    // transposed LDS writes of one instruction cover whole rows of V^T
    const bool v_active = tid < V_TASKS;
    const int v_kq = tid & 15;
    const int v_dc = tid >> 4;
    const int v_pos = (v_kq >> 2) * 16 + (v_kq & 1) * 8 + ((v_kq >> 1) & 1) * 4;

    uint4 kx[KT], ky[KT], vv[4];

    // Page ids are looked up one tile ahead of the loads that need them, so that the dependent
    // chain  block table -> page -> K/V row  never stalls a load: k_page[u] / v_page hold the pages of
    // the tile that the NEXT fetch_k / fetch_v call will read.  Columns past a conversation's last
    // page repeat a valid page of that row, so reading up to max_pages-1 is always in bounds.
    const int last_col = a.max_pages - 1;
    int k_page[KT], v_page;
#pragma unroll
    for (int u = 0; u < KT; ++u) k_page[u] = table[min(((tid + u * NTHREADS) / PIECES) >> 4, last_col)];
    v_page = table[min((4 * v_kq) >> 4, last_col)];

    // GUARD = false: the tile is known to lie entirely inside the visible keys (no bounds checks)
    auto fetch_k = [&](int tile, auto guard_tag) {   // HBM -> registers
        constexpr bool GUARD = decltype(guard_tag)::value;
        const int kt0 = tile * BN;
#pragma unroll
        for (int u = 0; u < KT; ++u) {
            const int task = tid + u * NTHREADS;
            const int t = kt0 + task / PIECES;
            if (GUARD) {
                kx[u] = make_uint4(0, 0, 0, 0);
                ky[u] = make_uint4(0, 0, 0, 0);
            }
            if ((K_TASKS % NTHREADS == 0 || task < K_TASKS) && (!GUARD || t < kmax)) {
                const uint16_t *krow = a.k_pool + (((int64_t)k_page[u] * Hkv + g) * kPageSize + (t & 15)) * D;
                kx[u] = *reinterpret_cast<const uint4 *>(krow + 8 * k_piece);
                ky[u] = *reinterpret_cast<const uint4 *>(krow + HALF + 8 * k_piece);
            }
            k_page[u] = table[min((t + BN) >> 4, last_col)];
        }
    };

    auto fetch_v = [&](int tile, auto guard_tag) {
        constexpr bool GUARD = decltype(guard_tag)::value;
        const int kt0 = tile * BN;
        if (v_active) {
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int t = kt0 + 4 * v_kq + rr;   // the 4 keys of a quad share a page
                if (GUARD) vv[rr] = make_uint4(0, 0, 0, 0);
                if (!GUARD || t < kmax) {
                    const uint16_t *vrow = a.v_pool + (((int64_t)v_page * Hkv + g) * kPageSize + (t & 15)) * D;
                    vv[rr] = *reinterpret_cast<const uint4 *>(vrow + 8 * v_dc);
                }
            }
            v_page = table[min((kt0 + BN + 4 * v_kq) >> 4, last_col)];
        }
    };

    // registers -> rotate -> LDS, then advance the rotation by one tile.  Cut into 4 parts (one per
    // dword of the two 16-byte pieces) so that the caller can spread the arithmetic between the
    // matrix instructions of the S^T product.
    auto stage_k_part = [&](int buf, int w) {
#pragma unroll
        for (int u = 0; u < KT; ++u) {
            const int task = tid + u * NTHREADS;
            if (K_TASKS % NTHREADS == 0 || task < K_TASKS) {
                uint32_t *pa = reinterpret_cast<uint32_t *>(&kx[u]);
                uint32_t *pb = reinterpret_cast<uint32_t *>(&ky[u]);
                const float a0 = bf_lo(pa[w]), a1 = bf_hi(pa[w]);
                const float b0 = bf_lo(pb[w]), b1 = bf_hi(pb[w]);
                if (STYLE == 0) {
                    const float2 c0 = k_cs[u][2 * w], c1 = k_cs[u][2 * w + 1];
                    pa[w] = pack_bf16(a0 * c0.x - b0 * c0.y, a1 * c1.x - b1 * c1.y);
                    pb[w] = pack_bf16(b0 * c0.x + a0 * c0.y, b1 * c1.x + a1 * c1.y);
                } else {
                    const float2 ca_ = k_cs[u][w], cb_ = k_cs[u][4 + w];
                    pa[w] = pack_bf16(a0 * ca_.x - a1 * ca_.y, a1 * ca_.x + a0 * ca_.y);
                    pb[w] = pack_bf16(b0 * cb_.x - b1 * cb_.y, b1 * cb_.x + b0 * cb_.y);
                }
#pragma unroll
                for (int e2 = 0; e2 < 2; ++e2) {
                    const int e = (STYLE == 0) ? 2 * w + e2 : w + 4 * e2;
                    const float2 o = k_cs[u][e], st = k_step[e];
                    k_cs[u][e] = make_float2(o.x * st.x - o.y * st.y, o.y * st.x + o.x * st.y);
                }
                if (w == 3) {
                    const int kk = task / PIECES;
                    *reinterpret_cast<uint4 *>(&Ks[buf][kk * KS_STRIDE + 8 * k_piece]) = kx[u];
                    *reinterpret_cast<uint4 *>(&Ks[buf][kk * KS_STRIDE + HALF + 8 * k_piece]) = ky[u];
                }
            }
        }
    };
    auto stage_k = [&](int buf) {
#pragma unroll
        for (int w = 0; w < 4; ++w) stage_k_part(buf, w);
    };

    auto stage_v = [&](int buf) {  // registers -> 4x8 transpose -> LDS as V^T
        // Inside a 16-key group the C layout of S^T hands P^T to the second product in the order
        // (half, e) <-> key (e/4)*8 + half*4 + e%4; V^T is stored in that order.
        if (v_active) {
            const uint32_t *w0 = reinterpret_cast<const uint32_t *>(&vv[0]);
            const uint32_t *w1 = reinterpret_cast<const uint32_t *>(&vv[1]);
            const uint32_t *w2 = reinterpret_cast<const uint32_t *>(&vv[2]);
            const uint32_t *w3 = reinterpret_cast<const uint32_t *>(&vv[3]);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                // dims 8dc + 2w (low halves) and 8dc + 2w + 1 (high halves)
                uint2 lo, hi;
                lo.x = __builtin_amdgcn_perm(w1[w], w0[w], 0x05040100u);
                lo.y = __builtin_amdgcn_perm(w3[w], w2[w], 0x05040100u);
                hi.x = __builtin_amdgcn_perm(w1[w], w0[w], 0x07060302u);
                hi.y = __builtin_amdgcn_perm(w3[w], w2[w], 0x07060302u);
                *reinterpret_cast<uint2 *>(&Vt[buf][(8 * v_dc + 2 * w) * VT_STRIDE + v_pos]) = lo;
                *reinterpret_cast<uint2 *>(&Vt[buf][(8 * v_dc + 2 * w + 1) * VT_STRIDE + v_pos]) = hi;
            }
        }
    };

    f32x16 O[DBLKS];
#pragma unroll
    for (int db = 0; db < DBLKS; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[db][i] = 0.f;
    float m_run = -INFINITY;   // reference maximum of the raw scores of this row (may lag, see above)
    float l_run = 0.f;         // this lane's share of the running denominator
    const float cscale = a.softmax_scale * 1.4426950408889634f;

    // One tile of the walk.  INTERIOR: the tile and the two after it are complete and no row of the
    // workgroup needs the causal mask on it, so the body is straight-line code the scheduler can
    // interleave (matrix products against the staging arithmetic); otherwise every step is guarded.
    // LIVE = false: this wavefront owns no valid row and only helps to stage tiles.
    auto walk = [&](int tile, auto interior_tag, auto live_tag) {
        constexpr bool INTERIOR = decltype(interior_tag)::value;
        constexpr bool LIVE = decltype(live_tag)::value;
        const int kt0 = tile * BN;
        const int buf = tile & 1;
        const bool compute = LIVE && (INTERIOR || kt0 <= wq_max);   // anything visible to this wavefront?

        f32x16 S[2];
        if (INTERIOR && LIVE) {
            // ---- S^T = K Q^T, with the staging of the next K tile spread between the matrix instructions --
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) S[mb][i] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(&Ks[buf][(32 * mb + lq) * KS_STRIDE + 16 * ks + 8 * half]);
                    S[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, Qf[ks], S[mb], 0, 0, 0);
                }
                if (ks % (KSTEPS / 4) == KSTEPS / 4 - 1) stage_k_part(buf ^ 1, ks / (KSTEPS / 4));
            }
            fetch_k(tile + 2, std::false_type{});
        } else {
            if (compute) {
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) S[mb][i] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb) {
                        const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(&Ks[buf][(32 * mb + lq) * KS_STRIDE + 16 * ks + 8 * half]);
                        S[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, Qf[ks], S[mb], 0, 0, 0);
                    }
            }
            // ---- producer: tile+1 from registers into the other LDS buffer (free since the last barrier),
            // and, the registers being free again, the loads of tile+2 start a whole tile ahead of their use
            if (INTERIOR || tile + 1 < n_tiles) stage_k(buf ^ 1);
            if (INTERIOR) fetch_k(tile + 2, std::false_type{});
            else if (tile + 2 < n_tiles) fetch_k(tile + 2, std::true_type{});
        }

        if (compute) {
            // ---- causal mask (only tiles that reach past the first row's horizon) -------------------
            if (!INTERIOR && kt0 + BN - 1 > wq_min) {
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = kt0 + 32 * mb + (i >> 2) * 8 + half * 4 + (i & 3);
                        if (key > qpos) S[mb][i] = -INFINITY;
                    }
            }

            // ---- online softmax with lazy rescaling --------------------------------------------------
            float mx = S[0][0];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, S[mb][i]);
            {   // lanes l and l+32 hold the two key halves of one query row: one swap gives both the other half
                const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
            }
            const bool raise = (mx - m_run) * cscale > 8.0f;   // also true on the first tile (m_run = -inf)
            if (__builtin_amdgcn_ballot_w64(raise) != 0) {
                const float m_new = raise ? mx : m_run;
                const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * cscale);
                m_run = m_new;
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < DBLKS; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) O[db][i] *= alpha;
            }
            const float mc = m_run * cscale;
            float psum = 0.f;
            // ---- P = exp2(S*c - m*c), 16 keys at a time, each chunk straight into O^T += V^T P^T -------
#pragma unroll
            for (int ks2 = 0; ks2 < 4; ++ks2) {
                const int mb = ks2 >> 1, kk2 = ks2 & 1;
                uint32_t pk[4];
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[mb][8 * kk2 + 2 * w], cscale, -mc));
                    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[mb][8 * kk2 + 2 * w + 1], cscale, -mc));
                    psum += p0 + p1;
                    pk[w] = pack_bf16(p0, p1);
                }
                const bf16x8 pb = __builtin_bit_cast(bf16x8, make_uint4(pk[0], pk[1], pk[2], pk[3]));
#pragma unroll
                for (int db = 0; db < DBLKS; ++db) {
                    const bf16x8 vf = *reinterpret_cast<const bf16x8 *>(&Vt[buf][(32 * db + lq) * VT_STRIDE + 16 * ks2 + 8 * half]);
                    O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb, O[db], 0, 0, 0);
                }
            }
            l_run += psum;
        }

        if (INTERIOR || tile + 1 < n_tiles) stage_v(buf ^ 1);
        if (INTERIOR) fetch_v(tile + 2, std::false_type{});
        else if (tile + 2 < n_tiles) fetch_v(tile + 2, std::true_type{});
        __syncthreads();   // tile+1 is complete in LDS; nobody still reads buffer `buf`
    };

    // ---- prologue: tile 0 into LDS, tile 1 into registers -------------------------------------------
    fetch_k(0, std::true_type{});
    fetch_v(0, std::true_type{});
    stage_k(0);
    stage_v(0);
    if (n_tiles > 1) { fetch_k(1, std::true_type{}); fetch_v(1, std::true_type{}); }
    __syncthreads();

    // interior tiles: fully visible to the first row of the workgroup, and tile+2 is a complete tile
    const int first_qpos = n + item.row0 / G;
    const int n_interior = max(0, min((first_qpos + 1) / BN, kmax / BN - 2));
    int tile = 0;
    if (wave_live) {
        for (; tile < n_interior; ++tile) walk(tile, std::true_type{}, std::true_type{});
        for (; tile < n_tiles; ++tile) walk(tile, std::false_type{}, std::true_type{});
    } else {
        for (; tile < n_interior; ++tile) walk(tile, std::true_type{}, std::false_type{});
        for (; tile < n_tiles; ++tile) walk(tile, std::false_type{}, std::false_type{});
    }

    // ---- epilogue: normalise and store --------------------------------------------------------------
    const float l_all = l_run + __shfl_xor(l_run, 32);
    if (row_valid) {
        const float inv = 1.f / l_all;
        uint16_t *orow = a.out + ((int64_t)(q0 + j) * a.n_q_heads + head) * D;
#pragma unroll
        for (int db = 0; db < DBLKS; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int d = 32 * db + i4 * 8 + half * 4;
                uint2 o;
                o.x = pack_bf16(O[db][4 * i4] * inv, O[db][4 * i4 + 1] * inv);
                o.y = pack_bf16(O[db][4 * i4 + 2] * inv, O[db][4 * i4 + 3] * inv);
                *reinterpret_cast<uint2 *>(orow + d) = o;
            }
    }
}

template <int NW>
hipError_t launch_nw(const AttnArgs &a, hipStream_t stream) {
    dim3 grid(a.n_items), block(64 * NW);
    if (a.head_dim == 128 && a.rope_style == 0)
        hipLaunchKernelGGL((attn_mfma_kernel<128, 0, NW>), grid, block, 0, stream, a);
    else if (a.head_dim == 128)
        hipLaunchKernelGGL((attn_mfma_kernel<128, 1, NW>), grid, block, 0, stream, a);
    else if (a.head_dim == 64 && a.rope_style == 0)
        hipLaunchKernelGGL((attn_mfma_kernel<64, 0, NW>), grid, block, 0, stream, a);
    else if (a.head_dim == 64)
        hipLaunchKernelGGL((attn_mfma_kernel<64, 1, NW>), grid, block, 0, stream, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_mfma(const AttnArgs &a, hipStream_t stream) {
    if (a.n_items <= 0) return hipSuccess;
    if (a.tile_rows == 128) return launch_nw<4>(a, stream);
    if (a.tile_rows == 256) return launch_nw<8>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace ca
