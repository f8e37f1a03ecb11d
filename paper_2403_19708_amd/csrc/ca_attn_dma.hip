// Fused rotary-on-load + causal varlen prefill attention (Sections 2.1, 3.1, 3.4) on the matrix cores.
//
// out[j, h, :] = sum_t softmax_t(RoPE(q[j,h], n+j) . RoPE(k[t], t) * scale) v[t] over the context tokens t <= n + j of
// the conversation, bf16 in, fp32 accumulate, bf16 out.  One workgroup = NW wavefronts x 32 stacked query rows (row r
// of a (conversation, kv head) <-> new token r / G, query head kv*G + r % G, so the G heads of a group share every
// staged K/V tile), walking key tiles of BN with an online softmax.  v_mfma_f32_32x32x16_bf16 in the transposed
// formulation S^T = K Q^T, O^T += V^T P^T: in the C layout a lane owns one query column, so row maxima and sums are
// in-lane plus one exchange with lane ^ 32, and the C registers of S^T, converted to bf16, ARE the B operand of the
// second product.  The softmax scale and log2(e) are folded into the rotated query before it is rounded to bf16 and the
// running reference maximum enters the score product as its initial accumulator (-m), so the exponent's argument comes
// straight out of the matrix instruction.  The reference maximum is raised lazily (a wave-uniform branch, rare after
// the first tile).
// K/V tiles travel HBM -> LDS without passing through registers:
//
//   * global_load_lds (16 bytes per lane, written to LDS at base + lane*16) fills a ring of 4 tile
//     stages in LDS; the loads of tile T+3 are issued when tile T starts, so two to three tiles
//     (64-96 KiB per compute unit) are in flight while one is multiplied, and no vector register
//     is spent on staging.  The only vector-memory instructions inside the walk are these loads,
//     so s_waitcnt vmcnt(N) with a constant N releases exactly the tile that is needed next.
//   * The page ids of the conversation are kept in LDS (a window of 2048 pages that follows the walk); the dependent chain
//     block table -> page -> row costs an LDS read.  On interior tiles a load's page and base address
//     are wave-uniform: all page ids of an iteration are read before the first is used (one LDS round
//     trip), and the scalar address arithmetic and the loads are issued after the first matrix
//     instructions of the tile, where they cost nothing.
//   * An item may own only a share [key_begin, key_end) of the keys its rows see (the host splits long
//     row tiles over several workgroups when a batch would otherwise leave compute units idle).  Such an
//     item leaves unnormalised sums, reference maxima and denominators in a scratch buffer and
//     combine_kernel merges the shares of a row tile.
//   * Since the LDS side of such a load is fixed (lane l -> byte l*16 of a 1 KiB chunk), the layout
//     is chosen on the global side: a chunk holds KPC = 1024/(2D) keys, piece-major
//     (slot = piece*KPC + key_in_chunk), chunks padded by KPC*16 bytes.  With it the A-operand reads
//     of K (32 keys x one 16-byte piece), the in-place rotary pass and the transposing reads of V
//     are all bank-conflict free, and the offset of a piece is linear in the piece index, so the
//     per-k-step offsets are instruction immediates.
//   * K lands in LDS without positions; the workgroup rotates the NEXT tile in place (LDS -> fp32
//     rotate -> bf16 -> same LDS bytes) while the matrix cores work on the current one.
//   * V is never transposed by the ALUs: ds_read_b64_tr_b16 hands each lane 4 consecutive keys of
//     one head dimension, which is exactly the A-operand layout of O^T += V^T P^T (two such reads
//     per operand, in the key order the C layout of S^T imposes on P^T).
//   * Keys past the end of the context are not zero-filled (a load cannot write zeros): the source
//     row is clamped to the last valid key, the causal mask gives those columns probability 0 and
//     the clamped V rows are finite data, so they contribute exactly nothing.
#include "ca_internal.h"

#include <type_traits>

namespace ca {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

constexpr int kMaxPagesLds = 2048;   // page ids kept in LDS at a time: a window of 32768 tokens that moves with the walk

__device__ inline float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ inline uint32_t pack_bf16(float a, float b) {
    bf16x2 v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(uint32_t, v);
}

// 16 bytes per lane, global -> LDS at lds_base + lane*16, no register in between.  Written as inline
// assembly on purpose: the compiler then knows nothing of the outstanding load and does not guard
// every later LDS read with s_waitcnt vmcnt(0) (it cannot tell which LDS bytes the load will write);
// the waits are placed by hand with CA_WAIT_VMCNT, which the in-order completion of these loads
// makes exact.  lds_base must be wave-uniform.
__device__ inline void dma16(const void *src, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_base), "v"(src) : "memory", "m0");
}

// same, with the address split into a wave-uniform 64-bit base (scalar registers) and a 32-bit
// per-lane byte offset: no vector arithmetic per load
__device__ inline void dma16_sbase(const void *base_uniform, uint32_t lane_off, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                 : : "s"(lds_base), "v"(lane_off), "s"(base_uniform) : "memory", "m0");
}

__device__ inline uint32_t lds_offset(const void *p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void *)p;
}

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt in bits 3:0 and
// 15:14, expcnt 6:4 and lgkmcnt 11:8 left at "don't wait")
#define CA_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

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

// one dword (2 elements) of each of the two 16-byte pieces a (dims d0..) and b (dims d0 + D/2..)
// (f = a factor applied to the rotated values before they are rounded)
template <int STYLE>
__device__ inline void rotate_dword(uint32_t &pa, uint32_t &pb, const float2 (&cs)[8], int w, float f = 1.0f) {
    const float a0 = bf_lo(pa), a1 = bf_hi(pa);
    const float b0 = bf_lo(pb), b1 = bf_hi(pb);
    if (STYLE == 0) {
        const float2 c0 = cs[2 * w], c1 = cs[2 * w + 1];
        pa = pack_bf16((a0 * c0.x - b0 * c0.y) * f, (a1 * c1.x - b1 * c1.y) * f);
        pb = pack_bf16((b0 * c0.x + a0 * c0.y) * f, (b1 * c1.x + a1 * c1.y) * f);
    } else {
        const float2 ca_ = cs[w], cb_ = cs[4 + w];
        pa = pack_bf16((a0 * ca_.x - a1 * ca_.y) * f, (a1 * ca_.x + a0 * ca_.y) * f);
        pb = pack_bf16((b0 * cb_.x - b1 * cb_.y) * f, (b1 * cb_.x + b0 * cb_.y) * f);
    }
}

// NW wavefronts (32 stacked query rows each) per workgroup, key tiles of BN.  Two shapes are built:
// NW = 8, BN = 64 (one workgroup per compute unit, 256-row tiles) and NW = 4, BN = 32 (two independent
// workgroups per compute unit, 128-row tiles: the two wavefronts that share a SIMD then belong to
// different workgroups, are not in lock step, and one's matrix products run under the other's softmax).
// ROT = false: the keys come already rotated from a scratch copy of the context (rotate_keys_kernel below),
// dense pages numbered per conversation; used when many row tiles share the keys of a (conversation, kv head)
// and rotating them once beats rotating them in every tile.
// NS = LDS stages of the tile ring: the loads of tile T+NS-1 go out in iteration T.
// PGW = page ids kept in LDS at a time, OCC = wavefronts per SIMD the register budget is cut for.
template <int D, int STYLE, int NW, int BN, bool ROT = true, int NS = 4, int PGW = kMaxPagesLds, int OCC = 2>
__global__ __launch_bounds__(64 * NW, OCC) void attn_dma_kernel(AttnArgs a) {
    static_assert(ROT ? NS >= 4 : NS >= 2, "the in-place rotary pass needs a tile landed one iteration early");
    constexpr int NTHREADS = 64 * NW;
    constexpr int MB = BN / 32;              // 32-key blocks of S^T per tile
    constexpr int KS2 = BN / 16;             // 16-key steps of the second product per tile
    constexpr int HALF = D / 2;
    constexpr int KSTEPS = D / 16;           // k-steps of the S^T product
    constexpr int DBLKS = D / 32;            // 32-row blocks of O^T
    constexpr int PPR = D / 8;               // 16-byte pieces per row
    constexpr int KPC = 64 / PPR;            // keys per 1 KiB chunk
    constexpr int CHUNKS = BN / KPC;         // chunks per K (or V) tile
    constexpr int CH = 1024 + KPC * 16;      // chunk stride in LDS (bytes)
    constexpr int TILE = CHUNKS * CH;        // bytes of one K (or V) tile in LDS
    constexpr int STAGE = 2 * TILE;
    constexpr int NI = 2 * CHUNKS / NW;      // load instructions per thread and tile (K and V)
    constexpr int ROT_TASKS = BN * PPR / 2;  // (key, piece pair) tasks of the rotary pass
    static_assert(2 * CHUNKS % NW == 0, "chunks divide evenly over the wavefronts");
    static_assert((NW == 8 ? 1 : OCC) * (NS * STAGE + PGW * 4) <= 160 * 1024, "LDS budget");
    // loads that may still be in flight at the end of an interior iteration: with the rotary pass tile+2 must have
    // landed (it is rotated next), without it only tile+1
    constexpr int FLY = ROT ? (NS > 3 ? NI : 0) : (NS - 2) * NI;

    __shared__ __attribute__((aligned(16))) uint8_t ring[NS * STAGE];
    __shared__ int32_t pg[PGW];

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
    // keys [key_begin, kmax): what the tile's rows can see, cut to the item's share when the keys of one
    // row tile are split over several workgroups (key_begin and a cutting key_end are multiples of 64)
    const int kmax = min(n + row_last / G + 1, item.key_end);
    const int t_begin = item.key_begin / BN;
    const int n_tiles = (kmax + BN - 1) / BN;                   // end of the walk (absolute tile index)

    // page ids of the visible context -> LDS, a window of kMaxPagesLds pages starting at the first tile's page; the
    // walk moves the window on when the loads it issues ahead would leave it (once per 32768 keys)
    const int n_pages = (kmax + kPageSize - 1) / kPageSize;
    int pg_base = t_begin * (BN / kPageSize);
    for (int i = tid; i < min(PGW, n_pages - pg_base); i += NTHREADS) pg[i] = table[pg_base + i];

    // ---- this lane's query row --------------------------------------------------------------
    const int r_raw = item.row0 + wave * 32 + lq;
    const bool row_valid = r_raw <= row_last;
    const int r = row_valid ? r_raw : row_last;
    const int j = r / G;
    const int head = g * G + (r - j * G);
    const int qpos = n + j;                                      // keys 0..qpos are visible
    const int wr_first = min(item.row0 + wave * 32, row_last);
    const int wr_last = min(item.row0 + wave * 32 + 31, row_last);
    const bool wave_live = item.row0 + wave * 32 <= row_last;
    const int wq_min = n + wr_first / G;
    const int wq_max = n + wr_last / G;

    // The softmax scale and log2(e) are folded into the rotated query before it is rounded to bf16, so the scores
    // come out of the matrix cores in the units of the base-2 exponent.
    const float cscale = a.softmax_scale * 1.4426950408889634f;
    bf16x8 Qf[KSTEPS];          // loaded and rotated in the prologue, once the first key/value tiles are on their way

    // ---- rotary pass: this thread's (key, piece pair) of every K tile ------------------------------
    const bool rot_active = ROT && (ROT_TASKS >= NTHREADS || tid < ROT_TASKS);
    // 16 consecutive lanes take the KPC keys of a chunk times consecutive pieces = 16 consecutive 16-byte
    // slots, so the 16-byte LDS accesses of the pass are free of bank conflicts (key-major lanes were 2-way)
    const int rot_kk = (tid / (KPC * (PPR / 2))) * KPC + tid % KPC;
    const int rot_pr = (tid / KPC) % (PPR / 2);
    const int rot_off = (rot_kk / KPC) * CH + (rot_pr * KPC + rot_kk % KPC) * 16;   // piece rot_pr; partner +512
    constexpr int ROT_PARTNER = (PPR / 2) * KPC * 16;
    float2 k_step[8], k_cs[8];
    if (ROT) load_cs<D, STYLE>(a.rope, BN, rot_pr, k_step);
    // first position of this thread's key; a thread whose first key lies past the visible range never sees a
    // visible one later either, so clamping it is harmless (and keeps the read inside the table)
    if (ROT) load_cs<D, STYLE>(a.rope, rot_active ? min(t_begin * BN + rot_kk, kmax - 1) : 0, rot_pr, k_cs);
    const uint16_t *const k_src = ROT ? a.k_pool : a.k_rot;
    const int k_page0 = ROT ? 0 : a.dense_page0[c];          // ROT = false: key page i of the conversation is k_page0 + i
    uint4 kx, ky;

    // ---- operand addresses inside a stage ---------------------------------------------------------------
    // K, A operand of S^T: key 32mb + lq, piece 2ks + half  ->  + ks * 2*KPC*16 as an immediate
    int k_rd[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int key = 32 * mb + lq;
        k_rd[mb] = (key / KPC) * CH + (half * KPC + key % KPC) * 16;
    }
    // V, A operand of O^T via transposing reads: lane s of a 16-lane group points at key k0 + s/4,
    // dims d0 + 4*(s%4) .. +3 and receives dims d0 + s of keys k0..k0+3
    const int s16 = lane & 15;
    const int dsel = (lane >> 4) & 1;
    int v_rd;
    {
        const int piece_lo = 2 * dsel + ((s16 & 3) >> 1);      // + 4*db
        const int kl = (D == 128) ? (s16 >> 2) : (4 * half + (s16 >> 2));
        v_rd = TILE + (piece_lo * KPC + kl) * 16 + (s16 & 1) * 8 + ((D == 128) ? half * CH : 0);
    }

    // ---- loads: chunk `wave + 8*i` of the 2*CHUNKS chunks [K | V] of a tile -----------------------------
    int ld_tok[NI], ld_goff[NI], ld_loff[NI];
    bool ld_is_v[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int cid = wave + NW * i;
        ld_is_v[i] = cid >= CHUNKS;
        const int jch = cid % CHUNKS;
        const int piece = lane / KPC, kl = lane % KPC;
        ld_tok[i] = jch * KPC + kl;                 // key inside the tile
        ld_goff[i] = piece * 8;                     // element offset inside the row
        ld_loff[i] = (ld_is_v[i] ? TILE : 0) + jch * CH;
    }
    auto issue = [&](int tile) {
        const int kt0 = tile * BN;
        uint8_t *stage = ring + (tile % NS) * STAGE;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int t = min(kt0 + ld_tok[i], kmax - 1);
            const int page = (ROT || ld_is_v[i]) ? pg[(t >> 4) - pg_base] : k_page0 + (t >> 4);
            const uint16_t *base = ld_is_v[i] ? a.v_pool : k_src;
            const uint16_t *src = base + (((int64_t)page * Hkv + g) * kPageSize + (t & 15)) * D + ld_goff[i];
            dma16(src, __builtin_amdgcn_readfirstlane(lds_offset(stage + ld_loff[i])));
        }
    };

    // Interior tiles need no clamping: all lanes of one load read rows of the same page, so the page
    // lookup and the whole address up to the lane's constant offset are wave-uniform (scalar ALU).
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t ld_lane_off = (uint32_t)((lane % KPC) * D + (lane / KPC) * 8) * 2u;
    auto issue_interior = [&](int tile) {
        const int kt0 = tile * BN;
        const uint32_t stage = __builtin_amdgcn_readfirstlane(lds_offset(ring)) + (uint32_t)((tile % NS) * STAGE);
        int page_v[NI];                     // all page ids first: one LDS round trip instead of NI
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int pi = (kt0 + ((wave_u + NW * i) % CHUNKS) * KPC) >> 4;
            page_v[i] = (ROT || wave_u + NW * i >= CHUNKS) ? pg[pi - pg_base] : k_page0 + pi;
        }
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int cid = wave_u + NW * i;
            const bool is_v = cid >= CHUNKS;
            const int jch = cid % CHUNKS;
            const int t0 = kt0 + jch * KPC;                                 // first key of the chunk
            const int page = __builtin_amdgcn_readfirstlane(page_v[i]);
            const uint16_t *base = (is_v ? a.v_pool : k_src) + (((int64_t)page * Hkv + g) * kPageSize + (t0 & 15)) * D;
            dma16_sbase(base, ld_lane_off, stage + (uint32_t)((is_v ? TILE : 0) + jch * CH));
        }
    };

    auto rot_read = [&](uint8_t *kst) {
        if (rot_active) {
            kx = *reinterpret_cast<const uint4 *>(kst + rot_off);
            ky = *reinterpret_cast<const uint4 *>(kst + rot_off + ROT_PARTNER);
        }
    };
    auto rot_part = [&](uint8_t *kst, int w) {
        if (rot_active) {
            uint32_t *pa = reinterpret_cast<uint32_t *>(&kx), *pb = reinterpret_cast<uint32_t *>(&ky);
            rotate_dword<STYLE>(pa[w], pb[w], k_cs, w);
#pragma unroll
            for (int e2 = 0; e2 < 2; ++e2) {
                const int e = (STYLE == 0) ? 2 * w + e2 : w + 4 * e2;
                const float2 o = k_cs[e], st = k_step[e];
                k_cs[e] = make_float2(o.x * st.x - o.y * st.y, o.y * st.x + o.x * st.y);
            }
            if (w == 3) {
                *reinterpret_cast<uint4 *>(kst + rot_off) = kx;
                *reinterpret_cast<uint4 *>(kst + rot_off + ROT_PARTNER) = ky;
            }
        }
    };

    f32x16 O[DBLKS];
#pragma unroll
    for (int db = 0; db < DBLKS; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[db][i] = 0.f;
    // m_run = reference maximum of this lane's query row in exponent units (-inf: no key seen yet); neg_m holds
    // -m_run (0 while there is none) in the C layout and is the accumulator input of the first matrix instruction
    // of every tile, so the scores arrive already relative to the reference and the common path of the softmax
    // is exp2 of the accumulator, with no subtraction per element
    float m_run = -INFINITY;
    float l_run = 0.f;
    f32x16 neg_m;
#pragma unroll
    for (int i = 0; i < 16; ++i) neg_m[i] = 0.f;
    const bf16x2 ones2 = {(__bf16)1.0f, (__bf16)1.0f};

    // ---- prologue ---------------------------------------------------------------------------------------
    __syncthreads();                     // page ids are in LDS
    issue(t_begin);
    if (NS > 2 && t_begin + 1 < n_tiles) issue(t_begin + 1);
    if (NS > 3 && t_begin + 2 < n_tiles) issue(t_begin + 2);
    // The query row is fetched behind the tile loads, so its latency and theirs overlap.  These loads are younger than
    // the tile loads and complete after them: the counted wait below can only become stricter by them.
    {
        const uint16_t *qrow = a.q + ((int64_t)(q0 + j) * a.n_q_heads + head) * D;
#pragma unroll
        for (int ks = 0; ks < KSTEPS / 2; ++ks) {
            const int piece = 2 * ks + half;
            uint4 x = *reinterpret_cast<const uint4 *>(qrow + 8 * piece);
            uint4 y = *reinterpret_cast<const uint4 *>(qrow + HALF + 8 * piece);
            float2 cs[8];
            load_cs<D, STYLE>(a.rope, qpos, piece, cs);
            uint32_t *px = reinterpret_cast<uint32_t *>(&x), *py = reinterpret_cast<uint32_t *>(&y);
#pragma unroll
            for (int w = 0; w < 4; ++w) rotate_dword<STYLE>(px[w], py[w], cs, w, cscale);
            Qf[ks] = __builtin_bit_cast(bf16x8, x);
            Qf[ks + KSTEPS / 2] = __builtin_bit_cast(bf16x8, y);
        }
    }
    if (NS > 3 && t_begin + 2 < n_tiles) { CA_WAIT_VMCNT(NI); } else { CA_WAIT_VMCNT(0); }   // the first two tiles have landed
    __syncthreads();
    rot_read(ring + (t_begin % NS) * STAGE);
#pragma unroll
    for (int w = 0; w < 4; ++w) rot_part(ring + (t_begin % NS) * STAGE, w);
    __syncthreads();

    auto walk = [&](int tile, auto interior_tag, auto live_tag) {
        constexpr bool INTERIOR = decltype(interior_tag)::value;
        constexpr bool LIVE = decltype(live_tag)::value;
        const int kt0 = tile * BN;
        // the loads issued in this iteration look up the pages of tile + NS - 1: move the page-id window when they
        // would fall outside it.  Every wavefront has left the previous iteration's lookups behind (barrier at its end).
        if ((tile + NS) * (BN / kPageSize) > pg_base + PGW) {
            pg_base = tile * (BN / kPageSize);
            for (int i = tid; i < min(PGW, n_pages - pg_base); i += NTHREADS) pg[i] = table[pg_base + i];
            __syncthreads();
        }
        uint8_t *st = ring + (tile % NS) * STAGE;
        uint8_t *st_next = ring + ((tile + 1) % NS) * STAGE;
        const bool compute = LIVE && (INTERIOR || kt0 <= wq_max);
        const bool has_next = INTERIOR || tile + 1 < n_tiles;

        // the stage multiplied in the previous iteration is free: refill it three tiles ahead
        // (interior tiles of wavefronts with rows issue a little later, under the first matrix instructions,
        // where the scalar address arithmetic costs nothing)
        if (INTERIOR && !LIVE) issue_interior(tile + NS - 1);
        else if (!INTERIOR && tile + NS - 1 < n_tiles) issue(tile + NS - 1);
        if (has_next) rot_read(st_next);

        f32x16 S[MB];
        if (compute) {
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(st + k_rd[mb] + ks * (2 * KPC * 16));
                    S[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, Qf[ks], ks == 0 ? neg_m : S[mb], 0, 0, 0);
                }
                if (INTERIOR && ks == 0) {
                    __builtin_amdgcn_sched_barrier(0);
                    issue_interior(tile + NS - 1);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (has_next && ks % (KSTEPS / 4) == KSTEPS / 4 - 1) rot_part(st_next, ks / (KSTEPS / 4));
            }
        } else if (has_next) {
#pragma unroll
            for (int w = 0; w < 4; ++w) rot_part(st_next, w);
        }

        if (compute) {
            if (!INTERIOR && kt0 + BN - 1 > wq_min) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = kt0 + 32 * mb + (i >> 2) * 8 + half * 4 + (i & 3);
                        if (key > qpos) S[mb][i] = -INFINITY;
                    }
            }
            float mx = S[0][0];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, S[mb][i]);
            {   // lanes l and l+32 hold the two key halves of one query row: one swap gives both the other half
                const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
            }
            // mx is relative to the reference.  The reference follows the maximum lazily: it moves when a row sees its
            // first key (whatever the value) or when a score exceeds it by more than 8 (probabilities up to 2^8 are
            // harmless in fp32 and bf16).  A row whose keys so far were all masked (possible when the keys of a row
            // tile are split) has mx = -inf and stays without a reference: its probabilities are exp2(-inf) = 0.
            const bool unseen = m_run == -INFINITY;
            const bool raise = mx > -INFINITY && (unseen || mx > 8.0f);
            if (__builtin_amdgcn_ballot_w64(raise) != 0) {
                const float delta = raise ? mx : 0.f;
                // (a first reference rescales nothing: the sums are still zero, and exp2(-delta) could overflow)
                const float alpha = (raise && !unseen) ? __builtin_amdgcn_exp2f(-delta) : 1.0f;
                if (raise) m_run = (unseen ? 0.f : m_run) + mx;
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < DBLKS; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) O[db][i] *= alpha;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) S[mb][i] -= delta;
                const float nm = (m_run == -INFINITY) ? 0.f : -m_run;
#pragma unroll
                for (int i = 0; i < 16; ++i) neg_m[i] = nm;
            }
            float psum = 0.f;
#pragma unroll
            for (int ks2 = 0; ks2 < KS2; ++ks2) {
                const int mb = ks2 >> 1, kk2 = ks2 & 1;
                uint32_t pk[4];
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float p0 = __builtin_amdgcn_exp2f(S[mb][8 * kk2 + 2 * w]);
                    const float p1 = __builtin_amdgcn_exp2f(S[mb][8 * kk2 + 2 * w + 1]);
                    pk[w] = pack_bf16(p0, p1);
                    // the denominator sums the rounded probabilities, the very values the second product uses
                    psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk[w]), ones2, psum, false);
                }
                const bf16x8 pb = __builtin_bit_cast(bf16x8, make_uint4(pk[0], pk[1], pk[2], pk[3]));
#pragma unroll
                for (int db = 0; db < DBLKS; ++db) {
                    // keys 16ks2 + 4half + 0..3 and 16ks2 + 8 + 4half + 0..3 of dims 32db + lq
                    constexpr int KEY_STEP = (D == 128) ? 1 : 0;   // D = 128: 4 keys per chunk, a quad is a chunk
                    const int o0 = (D == 128 ? (4 * ks2) * CH : (2 * ks2) * CH) + 4 * db * KPC * 16;
                    const int o1 = (D == 128 ? (4 * ks2 + 2) * CH : (2 * ks2 + 1) * CH) + 4 * db * KPC * 16;
                    (void)KEY_STEP;
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(st + v_rd + o0));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(st + v_rd + o1));
                    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pb, O[db], 0, 0, 0);
                }
            }
            l_run += psum;
        }

        // tile+2 must have landed before anyone rotates it in the next iteration; the loads of tile+3
        // (issued at the top of this iteration) may stay in flight
        if (INTERIOR) { CA_WAIT_VMCNT(FLY); } else { CA_WAIT_VMCNT(0); }
        __syncthreads();
    };

    const int first_qpos = n + item.row0 / G;
    const int n_interior = max(t_begin, min((first_qpos + 1) / BN, kmax / BN - NS));   // end of the interior tiles
    int tile = t_begin;
    if (wave_live) {
        for (; tile < n_interior; ++tile) walk(tile, std::true_type{}, std::true_type{});
        for (; tile < n_tiles; ++tile) walk(tile, std::false_type{}, std::true_type{});
    } else {
        for (; tile < n_interior; ++tile) walk(tile, std::true_type{}, std::false_type{});
        for (; tile < n_tiles; ++tile) walk(tile, std::false_type{}, std::false_type{});
    }

    // ---- epilogue: normalise and store --------------------------------------------------------------
    const float l_all = l_run + __shfl_xor(l_run, 32);
    if (item.part >= 0) {
        // keys split over several workgroups: leave the unnormalised sums, the reference maximum and the
        // denominator of this share in the scratch buffer; combine_kernel merges the shares
        if (row_valid) {
            const int rt = r - item.row0;                       // row inside the tile
            float *base = a.partial + (int64_t)item.part * a.tile_rows * (D + 2);
            float *prow = base + (int64_t)rt * D;
#pragma unroll
            for (int db = 0; db < DBLKS; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const int d = 32 * db + i4 * 8 + half * 4;
                    *reinterpret_cast<float4 *>(prow + d) = make_float4(O[db][4 * i4], O[db][4 * i4 + 1], O[db][4 * i4 + 2], O[db][4 * i4 + 3]);
                }
            if (half == 0) {
                base[(int64_t)a.tile_rows * D + rt] = m_run / cscale;      // combine_kernel takes it in score units
                base[(int64_t)a.tile_rows * (D + 1) + rt] = l_all;
            }
        }
        return;
    }
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

// Merges the shares of row tiles whose keys were split (Section 2.1's softmax over the union of the key
// ranges): with M = max_s m_s and w_s = exp2((m_s - M) * c), out = sum_s w_s O_s / sum_s w_s l_s.
// blockIdx.x = split row tile, blockIdx.y = group of 256 / (D/4) rows; a thread owns four head dimensions of
// one row and has the loads of all shares in flight at once.
__global__ __launch_bounds__(256) void combine_kernel(AttnArgs a) {
    const CombineItem ci = a.combine[blockIdx.x];
    const int D = a.head_dim;
    const int vec_per_row = D / 4;
    const int rt = blockIdx.y * (256 / vec_per_row) + threadIdx.x / vec_per_row;
    if (rt >= ci.n_rows) return;
    const int d = 4 * (threadIdx.x % vec_per_row);
    const int G = a.n_q_heads / a.n_kv_heads;
    const float cscale = a.softmax_scale * 1.4426950408889634f;
    const int64_t part_stride = (int64_t)a.tile_rows * (D + 2);
    const float *first = a.partial + ci.first_part * part_stride;
    float m[kAttnMaxPartsPerTile], l[kAttnMaxPartsPerTile];
    float4 o[kAttnMaxPartsPerTile];
#pragma unroll
    for (int s = 0; s < kAttnMaxPartsPerTile; ++s) {
        const bool on = s < ci.n_parts;
        const float *base = first + (on ? s : 0) * part_stride;
        m[s] = on ? base[(int64_t)a.tile_rows * D + rt] : -INFINITY;
        l[s] = base[(int64_t)a.tile_rows * (D + 1) + rt];
        o[s] = *reinterpret_cast<const float4 *>(base + (int64_t)rt * D + d);
    }
    float M = m[0];
#pragma unroll
    for (int s = 1; s < kAttnMaxPartsPerTile; ++s) M = fmaxf(M, m[s]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float lsum = 0.f;
#pragma unroll
    for (int s = 0; s < kAttnMaxPartsPerTile; ++s) {
        const float w = (m[s] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m[s] - M) * cscale);
        acc.x += w * o[s].x; acc.y += w * o[s].y; acc.z += w * o[s].z; acc.w += w * o[s].w;
        lsum += w * l[s];
    }
    const float inv = 1.f / lsum;
    const int r = ci.row0 + rt;
    const int j = r / G;
    const int head = ci.kv_head * G + (r - j * G);
    uint2 ob;
    ob.x = pack_bf16(acc.x * inv, acc.y * inv);
    ob.y = pack_bf16(acc.z * inv, acc.w * inv);
    *reinterpret_cast<uint2 *>(a.out + ((int64_t)(a.cu_q[ci.seq] + j) * a.n_q_heads + head) * D + d) = ob;
}

// Rotates the keys of the whole batch context once (Section 3.4: the rebased positional encoding, applied
// when the cache is used): dense page dp of the scratch copy = pool page rot_src_page[dp] with token slot s
// rotated at position rot_pos0[dp] + s, in fp32 from the table, rounded to bf16 -- the same values the fused
// path forms tile by tile (there with the rotation advanced by recurrence).  one workgroup per (dense page, kv head);
// a thread owns one (token, pair of 16-byte pieces).  Slots past the end of a context hold whatever the pool
// holds; nobody reads them.
template <int D, int STYLE>
__global__ __launch_bounds__(D) void rotate_keys_kernel(AttnArgs a) {
    constexpr int HALF = D / 2;
    constexpr int PAIRS = D / 16;                       // piece pairs per row
    static_assert(kPageSize * PAIRS == D, "one thread per (token of the page, piece pair)");
    // workgroup i runs on die i % 8: the heads of a page go to one die, one after the other, because they
    // read the same 16 rows of the rotary table (its L2 then serves seven of the eight reads)
    const int die = blockIdx.x % 8, k = blockIdx.x / 8;
    const int dp = (k / a.n_kv_heads) * 8 + die, g = k % a.n_kv_heads;
    if (dp >= a.n_dense_pages) return;
    const int key = threadIdx.x / PAIRS, pr = threadIdx.x % PAIRS;
    if (key >= kPageSize) return;
    const int pos = min(a.rot_pos0[dp] + key, a.max_positions - 1);
    const int64_t src = (((int64_t)a.rot_src_page[dp] * a.n_kv_heads + g) * kPageSize + key) * D;
    const int64_t dst = (((int64_t)dp * a.n_kv_heads + g) * kPageSize + key) * D;
    uint4 x = *reinterpret_cast<const uint4 *>(a.k_pool + src + 8 * pr);
    uint4 y = *reinterpret_cast<const uint4 *>(a.k_pool + src + HALF + 8 * pr);
    float2 cs[8];
    load_cs<D, STYLE>(a.rope, pos, pr, cs);
    uint32_t *px = reinterpret_cast<uint32_t *>(&x), *py = reinterpret_cast<uint32_t *>(&y);
#pragma unroll
    for (int w = 0; w < 4; ++w) rotate_dword<STYLE>(px[w], py[w], cs, w);
    *reinterpret_cast<uint4 *>(a.k_rot + dst + 8 * pr) = x;
    *reinterpret_cast<uint4 *>(a.k_rot + dst + HALF + 8 * pr) = y;
}

template <int NW, int BN>
hipError_t launch_shape(const AttnArgs &a, hipStream_t stream) {
    dim3 grid(a.n_items), block(64 * NW);
    if (a.head_dim == 128 && a.rope_style == 0)
        hipLaunchKernelGGL((attn_dma_kernel<128, 0, NW, BN>), grid, block, 0, stream, a);
    else if (a.head_dim == 128)
        hipLaunchKernelGGL((attn_dma_kernel<128, 1, NW, BN>), grid, block, 0, stream, a);
    else if (a.head_dim == 64 && a.rope_style == 0)
        hipLaunchKernelGGL((attn_dma_kernel<64, 0, NW, BN>), grid, block, 0, stream, a);
    else if (a.head_dim == 64)
        hipLaunchKernelGGL((attn_dma_kernel<64, 1, NW, BN>), grid, block, 0, stream, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_dma(const AttnArgs &a, hipStream_t stream) {
    if (a.n_items <= 0) return hipSuccess;
    if (a.n_combine > 0 && (a.partial == nullptr || a.combine == nullptr)) return hipErrorInvalidValue;
    hipError_t e;
    if (a.prerotate) {
        if ((a.tile_rows != 256 && a.tile_rows != 128) || !a.k_rot || !a.dense_page0 || !a.rot_src_page || !a.rot_pos0 || a.n_dense_pages <= 0)
            return hipErrorInvalidValue;
        const dim3 rgrid((uint32_t)((a.n_dense_pages + 7) / 8) * 8u * (uint32_t)a.n_kv_heads), grid(a.n_items);
        const bool big = a.tile_rows == 256;
#define CA_LAUNCH_PREROT(DD, ST)                                                                              \
        do {                                                                                                  \
            hipLaunchKernelGGL((rotate_keys_kernel<DD, ST>), rgrid, dim3(DD), 0, stream, a);                 \
            if (big) hipLaunchKernelGGL((attn_dma_kernel<DD, ST, 8, 64, false>), grid, dim3(512), 0, stream, a); \
            else hipLaunchKernelGGL((attn_dma_kernel<DD, ST, 4, 32, false>), grid, dim3(256), 0, stream, a);  \
        } while (0)
        if (a.head_dim == 128 && a.rope_style == 0) CA_LAUNCH_PREROT(128, 0);
        else if (a.head_dim == 128) CA_LAUNCH_PREROT(128, 1);
        else if (a.head_dim == 64 && a.rope_style == 0) CA_LAUNCH_PREROT(64, 0);
        else if (a.head_dim == 64) CA_LAUNCH_PREROT(64, 1);
        else return hipErrorInvalidValue;
#undef CA_LAUNCH_PREROT
        e = hipGetLastError();
    } else if (a.tile_rows == 256) e = launch_shape<8, 64>(a, stream);
    else if (a.tile_rows == 128) e = launch_shape<4, 32>(a, stream);
    else return hipErrorInvalidValue;
    if (e != hipSuccess || a.n_combine <= 0) return e;
    return launch_attn_combine(a, stream);
}

hipError_t launch_attn_combine(const AttnArgs &a, hipStream_t stream) {
    if (a.n_combine <= 0) return hipSuccess;
    if (a.partial == nullptr || a.combine == nullptr) return hipErrorInvalidValue;
    const int rows_per_group = 256 / (a.head_dim / 4);
    hipLaunchKernelGGL(combine_kernel, dim3(a.n_combine, (a.tile_rows + rows_per_group - 1) / rows_per_group), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace ca
