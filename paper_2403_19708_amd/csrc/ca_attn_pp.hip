// Causal varlen prefill attention of the new tokens over [kept history | new tokens] (Sections 2.1, 3.1,
// 3.4) for batches in which many row tiles share the keys of a (conversation, kv head) -- long new turns
// with grouped query heads, the matrix-core-bound case.  Two kernels:
//
//   prepare_kv_kernel   once per layer and batch: writes a scratch copy of the batch's context in the layout
//                       the matrix instructions want.  Keys: rotated at their rebased positions (the
//                       positional encoding of Section 3.4, applied when the cache is used), each (page, head)
//                       block stored piece-major, [16 pieces of 8 dims][16 keys][8 dims].  Values: each
//                       (page, head) block transposed, [2 key halves][128 dims][8 keys], the 8 keys of half h
//                       being slots 4h..4h+3 and 8+4h..8+4h+3 of the page.  Slots past the end of a context
//                       are written as zeros.  The pool itself is not modified.
//   attn_pp_kernel      8 wavefronts x 32 stacked query rows per workgroup, key tiles of 64, the same transposed
//                       products as the other kernels (S^T = K Q^T, O^T += V^T P^T, v_mfma_f32_32x32x16_bf16),
//                       software pipelined inside every wavefront:
//
// * Every operand of either product is ONE 16-byte LDS read whose 16-lane groups touch 256 consecutive
//   bytes (no bank conflicts, no transposing reads): that is what the two scratch layouts are for.  A block
//   is 4 KiB contiguous in memory and lands in LDS unchanged, 1 KiB per global_load_lds instruction; no page
//   table is needed (the scratch pages of a conversation are consecutive), hence no limit on the window, and no
//   padding.
// * While the matrix cores form the scores of tile T + 1 and the value product of tile T, the vector ALU takes
//   the softmax of tile T: the 32 matrix instructions of a tile are written as 32 inline-assembly chunks (wait for
//   the operand, matrix instruction, LDS read of the operand six instructions ahead) and the row maximum, the lazy
//   rescale decision and the exponentials sit between the chunks, two probabilities per chunk, in the order the
//   value product consumes them.  Two score buffers swap roles from tile to tile.  Measured on the chip: a
//   wavefront issues a matrix instruction every 32 cycles at best, and four to six vector instructions plus an
//   LDS read fit in between at no cost.
// * One barrier per tile (the K/V ring); keys are requested four tiles ahead, values three, into separate rings of
//   four 16 KiB slots.
// * The softmax scale and log2(e) are folded into the rotated query before it is rounded to bf16.
//
// What it buys: nothing in time on the workloads measured (config 5: 1.8 ms per launch, as the lock-step kernel),
// and the transposing pre-pass costs 0.13 ms more; three schedules of this arithmetic (lock step, two alternating
// groups of wavefronts, this one) land within a few per cent of each other, and switching any one ingredient off
// (vector work, LDS reads, loads, barrier) shortens the kernel by about that ingredient's own time: the parts do
// not hide behind each other.  Kept selectable (attn_schedule = 1) because it has no window limit.
#include "ca_internal.h"

namespace ca {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kD = 128;                  // head dimension this kernel is built for
constexpr int kBN = 64;                  // keys per tile
constexpr int kNW = 8;                   // wavefronts per workgroup
constexpr int kBlock = kPageSize * kD * 2;   // bytes of one (page, head) block: 4096
constexpr int kTile = (kBN / kPageSize) * kBlock;   // bytes of one K (or V) tile: 16384
constexpr int kNS = 4;                   // ring slots per array
#ifndef CA_PP_AHEAD
#define CA_PP_AHEAD 8
#endif
constexpr int kAhead = CA_PP_AHEAD;      // LDS operand reads in flight ahead of the matrix instruction that uses them

__device__ inline float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ inline uint32_t pack_bf16(float a, float b) {
    bf16x2 v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(uint32_t, v);
}

// 16 bytes per lane, global -> LDS at lds_base + lane*16, address = wave-uniform 64-bit base + per-lane byte
// offset.  Inline assembly so that the compiler does not guard later LDS reads with s_waitcnt vmcnt(0); the
// waits are placed by hand (these loads complete in order).
__device__ inline void dma16_sbase(const void *base_uniform, uint32_t lane_off, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                 : : "s"(lds_base), "v"(lane_off), "s"(base_uniform) : "memory", "m0");
}

__device__ inline uint32_t lds_offset(const void *p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void *)p;
}

#define CA_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

// (cos, sin) of the 8 pairs a thread rotates: STYLE 0 pairs (d, d + 64) of piece `piece` (dims 8*piece ..) and
// its partner piece + 8; STYLE 1 pairs (2i, 2i+1) inside piece `piece` (cs[0..3]) and inside piece + 8 (cs[4..7])
template <int STYLE>
__device__ inline void load_cs(const float2 *__restrict__ rope, int pos, int piece, float2 (&cs)[8]) {
    constexpr int HALF = kD / 2;
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

// one dword (2 elements) of each of the two 16-byte pieces a (dims d0..) and b (dims d0 + 64..), times `scale`
template <int STYLE>
__device__ inline void rotate_dword(uint32_t &pa, uint32_t &pb, const float2 (&cs)[8], int w, float scale) {
    const float a0 = bf_lo(pa), a1 = bf_hi(pa);
    const float b0 = bf_lo(pb), b1 = bf_hi(pb);
    if (STYLE == 0) {
        const float2 c0 = cs[2 * w], c1 = cs[2 * w + 1];
        pa = pack_bf16((a0 * c0.x - b0 * c0.y) * scale, (a1 * c1.x - b1 * c1.y) * scale);
        pb = pack_bf16((b0 * c0.x + a0 * c0.y) * scale, (b1 * c1.x + a1 * c1.y) * scale);
    } else {
        const float2 ca_ = cs[w], cb_ = cs[4 + w];
        pa = pack_bf16((a0 * ca_.x - a1 * ca_.y) * scale, (a1 * ca_.x + a0 * ca_.y) * scale);
        pb = pack_bf16((b0 * cb_.x - b1 * cb_.y) * scale, (b1 * cb_.x + b0 * cb_.y) * scale);
    }
}

// ---------------------------------------------------------------------------------------------------------
// scratch copy of the batch context: rotated keys (piece-major blocks) and transposed values
// ---------------------------------------------------------------------------------------------------------
// one workgroup of 256 threads per (dense page, kv head).  Workgroup i runs on die i % 8: the heads of a page go
// to one die, one after the other, because they read the same 16 rows of the rotary table.
template <int STYLE>
__global__ __launch_bounds__(256) void prepare_kv_kernel(AttnArgs a) {
    constexpr int HALF = kD / 2;
    const int die = blockIdx.x % 8, k = blockIdx.x / 8;
    const int dp = (k / a.n_kv_heads) * 8 + die, g = k % a.n_kv_heads;
    if (dp >= a.n_dense_pages) return;
    const int tid = threadIdx.x;
    const int nvalid = a.rot_nvalid[dp];
    const int64_t src = ((int64_t)a.rot_src_page[dp] * a.n_kv_heads + g) * kPageSize * kD;   // elements
    const int64_t dst = ((int64_t)dp * a.n_kv_heads + g) * kPageSize * kD;
    if (tid < 128) {
        // keys: thread = (slot, pair of pieces pr and pr + 8)
        const int key = tid >> 3, pr = tid & 7;
        uint4 x = make_uint4(0, 0, 0, 0), y = make_uint4(0, 0, 0, 0);
        if (key < nvalid) {
            const int pos = min(a.rot_pos0[dp] + key, a.max_positions - 1);
            x = *reinterpret_cast<const uint4 *>(a.k_pool + src + key * kD + 8 * pr);
            y = *reinterpret_cast<const uint4 *>(a.k_pool + src + key * kD + HALF + 8 * pr);
            float2 cs[8];
            load_cs<STYLE>(a.rope, pos, pr, cs);
            uint32_t *px = reinterpret_cast<uint32_t *>(&x), *py = reinterpret_cast<uint32_t *>(&y);
#pragma unroll
            for (int w = 0; w < 4; ++w) rotate_dword<STYLE>(px[w], py[w], cs, w, 1.0f);
        }
        // piece-major block: piece p, slot s at element (p * 16 + s) * 8
        *reinterpret_cast<uint4 *>(a.k_rot + dst + (pr * kPageSize + key) * 8) = x;
        *reinterpret_cast<uint4 *>(a.k_rot + dst + ((pr + 8) * kPageSize + key) * 8) = y;
    }
    {
        // values: thread = (key half h, dim d) gathers slots 4h..4h+3, 8+4h..8+4h+3 of dim d
        const int h = tid >> 7, d = tid & 127;
        uint16_t v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int slot = (i < 4) ? 4 * h + i : 8 + 4 * h + (i - 4);
            v[i] = slot < nvalid ? a.v_pool[src + slot * kD + d] : (uint16_t)0;
        }
        uint4 o;
        o.x = v[0] | ((uint32_t)v[1] << 16);
        o.y = v[2] | ((uint32_t)v[3] << 16);
        o.z = v[4] | ((uint32_t)v[5] << 16);
        o.w = v[6] | ((uint32_t)v[7] << 16);
        *reinterpret_cast<uint4 *>(a.v_t + dst + (h * kD + d) * 8) = o;
    }
}

// ---------------------------------------------------------------------------------------------------------
// the attention kernel
// ---------------------------------------------------------------------------------------------------------
// element i (0..31) of the scores of the tile whose softmax is being taken: two 32x32 blocks of S^T
#define SC(i) ((i) < 16 ? Sc0[(i)] : Sc1[(i) - 16])

template <int STYLE>
__global__ __launch_bounds__(64 * kNW, 2) void attn_pp_kernel(AttnArgs a) {
    constexpr int HALF = kD / 2;
    constexpr int KSTEPS = kD / 16;          // 8 k-steps of the score product
    constexpr int DBLKS = kD / 32;           // 4 blocks of 32 output dims

    __shared__ __attribute__((aligned(16))) uint8_t kring[kNS * kTile];
    __shared__ __attribute__((aligned(16))) uint8_t vring[kNS * kTile];

    const WorkItem item = a.items[blockIdx.x];
    if (item.seq < 0) return;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int lq = lane & 31;
    const int half = lane >> 5;

    const int c = item.seq;
    const int g = item.kv_head;
    const int G = a.n_q_heads / a.n_kv_heads;
    const int n = a.n_keep[c];
    const int q0 = a.cu_q[c];
    const int ctx_len = n + (a.cu_q[c + 1] - q0);
    const int last_page = (ctx_len - 1) / kPageSize;                  // last scratch page of the conversation
    const int Hkv = a.n_kv_heads;

    const int row_last = item.row0 + item.n_rows - 1;
    const int kmax = min(n + row_last / G + 1, item.key_end);          // keys [key_begin, kmax) are this item's
    const int t_begin = item.key_begin / kBN;
    const int n_tiles = (kmax + kBN - 1) / kBN;                       // absolute index one past the last tile

    // ---- this lane's query row ------------------------------------------------------------------------------
    const int r_raw = item.row0 + wave * 32 + lq;
    const bool row_valid = r_raw <= row_last;
    const int r = row_valid ? r_raw : row_last;
    const int j = r / G;
    const int head = g * G + (r - j * G);
    const int qpos = n + j;                                           // keys 0..qpos are visible
    const int wr_first = min(item.row0 + wave * 32, row_last);
    const int wq_min = n + wr_first / G;
    // tiles below w_full are seen whole by every row of this wavefront: no mask
    const int w_full = min((wq_min + 1) / kBN, kmax / kBN);

    const float cscale = a.softmax_scale * 1.4426950408889634f;   // exponent arguments come in units of log2

    // ---- operand addresses inside a tile -----------------------------------------------------------------------
    // K, A operand of S^T, block mb (32 keys = 2 pages), k-step ks: key 32mb + lq, piece 2ks + half
    //   -> (2mb + lq/16) * 4096 + (2ks + half) * 256 + (lq % 16) * 16
    const int k_rd = (lq >> 4) * kBlock + half * 256 + (lq & 15) * 16;            // + mb * 8192 + ks * 512
    // V^T, A operand of O^T, k-step ks2 (= page ks2 of the tile), dims 32db + lq, key half `half`
    //   -> ks2 * 4096 + half * 2048 + (32db + lq) * 16
    const int v_rd = half * 2048 + lq * 16;                                       // + ks2 * 4096 + db * 512

    // ---- loads: this wavefront moves quarter blocks wave and wave + 8 of the 16 of a K tile, and of a V tile -------
    const int64_t blk_stride = (int64_t)Hkv * kBlock;                               // bytes from one scratch page to the next
    const uint8_t *k_base = reinterpret_cast<const uint8_t *>(a.k_rot) + ((int64_t)a.dense_page0[c] * Hkv + g) * kBlock;
    const uint8_t *v_base = reinterpret_cast<const uint8_t *>(a.v_t) + ((int64_t)a.dense_page0[c] * Hkv + g) * kBlock;
    const uint32_t lane_off = (uint32_t)lane * 16u;
    const uint32_t kring0 = __builtin_amdgcn_readfirstlane(lds_offset(kring));
    const uint32_t vring0 = __builtin_amdgcn_readfirstlane(lds_offset(vring));
    auto issue_tile = [&](const uint8_t *base, uint32_t ring0, int tile) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int idx = wave + kNW * i;                       // quarter block of the tile: page idx / 4, quarter idx % 4
            const int page = min(tile * (kBN / kPageSize) + (idx >> 2), last_page);   // pages past the context: masked keys, finite data
            const uint8_t *src = base + (int64_t)page * blk_stride + (idx & 3) * 1024;
            dma16_sbase(src, lane_off, ring0 + (uint32_t)((tile % kNS) * kTile + idx * 1024));
        }
    };

    bf16x8 Qf[KSTEPS];                    // this lane's query row, B operand of the score product (filled in the prologue)
    f32x16 O[DBLKS];
#pragma unroll
    for (int db = 0; db < DBLKS; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[db][i] = 0.f;
    f32x16 Sa0, Sa1, Sb0, Sb1;            // scores of two tiles in flight: one being exponentiated, one being multiplied
    float M = 0.f;                        // reference maximum (log2 units); meaningless until `seen`
    bool seen = false;                    // the row has met a visible key
    float l_run = 0.f;
    uint32_t Pk[16];                      // probabilities of the current tile, bf16 pairs: B operand of O^T += V^T P^T
    const bf16x2 ones2 = {(__bf16)1.0f, (__bf16)1.0f};
    bf16x8 t0, t1, t2, t3, t4, t5, t6, t7;   // ring of LDS operand registers

    // the reference is raised lazily: on the row's first visible key, and when a score exceeds it by 2^8
#define RAISE_CHECK(mx)                                                                                            \
    do {                                                                                                           \
        const bool raise = (mx) > -INFINITY && (!seen || (mx) - M > 8.0f);                                         \
        if (__builtin_amdgcn_ballot_w64(raise) != 0) {                                                             \
            const float alpha = (raise && seen) ? __builtin_amdgcn_exp2f(M - (mx)) : 1.0f;                         \
            M = raise ? (mx) : M;                                                                                  \
            seen = seen || raise;                                                                                  \
            l_run *= alpha;                                                                                        \
            _Pragma("unroll") for (int db = 0; db < DBLKS; ++db)                                                   \
                _Pragma("unroll") for (int i = 0; i < 16; ++i) O[db][i] *= alpha;                                  \
        }                                                                                                          \
    } while (0)
    // two probabilities: exponent, rounded to bf16 for the second product; the denominator sums the rounded values
#define SOFTMAX_PAIR(e)                                                                                            \
    do {                                                                                                           \
        const float p0 = __builtin_amdgcn_exp2f(SC(2 * (e)) - M), p1 = __builtin_amdgcn_exp2f(SC(2 * (e) + 1) - M); \
        const uint32_t pk = pack_bf16(p0, p1);                                                                     \
        Pk[(e)] = pk;                                                                                              \
        psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), ones2, psum, false);                \
    } while (0)

    // One key tile, software pipelined inside the wavefront: the 16 matrix instructions of the NEXT tile's scores
    // (into Sn) and the 16 of THIS tile's value product, in this order, each as one inline-assembly chunk
    //   s_waitcnt (its operand has landed) ; v_mfma ; ds_read (the operand of the instruction six further on)
    // with the vector-ALU work of this tile's softmax (on Sc, finished a tile ago) in the chunks' shadow: row maximum
    // under the first seven, the lazy rescale decision under the eighth, then two probabilities per chunk, so that
    // the k-step of the value product that needs them finds them ready.  A wavefront issues a matrix instruction
    // every 32 cycles at best, four to six vector instructions and an LDS read fit in between for free (measured);
    // the two wavefronts of a SIMD run this unsynchronised apart from one barrier per tile, and whatever one leaves of
    // the matrix pipe the other takes.  The operand ring has eight registers: a read never targets the register of
    // the previous two matrix instructions.  sched_barrier keeps the compiler from moving the vector work across chunks.
    auto tile_block = [&](f32x16 &Sc0, f32x16 &Sc1, f32x16 &Sn0, f32x16 &Sn1, int T, bool masked) {
        const uint32_t ka = lds_offset(kring + ((T + 1) % kNS) * kTile + k_rd);
        const uint32_t va = lds_offset(vring + (T % kNS) * kTile + v_rd);
        if (masked) {
            const int kt0 = T * kBN;
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                const int key = kt0 + 32 * (i >> 4) + ((i & 15) >> 2) * 8 + half * 4 + (i & 3);
                if (key > qpos || key >= kmax) { if (i < 16) Sc0[i & 15] = -INFINITY; else Sc1[i & 15] = -INFINITY; }
            }
        }
        float psum = 0.f;
        {
// ---- GENERATED by the development helper gen_tile_block.py: 32 chunks ----
            // first operands of the tile
            asm volatile(
                "ds_read_b128 %[t0], %[ka] offset:0\n\t"
                "ds_read_b128 %[t1], %[ka] offset:8192\n\t"
                "ds_read_b128 %[t2], %[ka] offset:512\n\t"
                "ds_read_b128 %[t3], %[ka] offset:8704\n\t"
                "ds_read_b128 %[t4], %[ka] offset:1024\n\t"
                "ds_read_b128 %[t5], %[ka] offset:9216\n\t"
                : [t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2), [t3] "=&v"(t3), [t4] "=&v"(t4), [t5] "=&v"(t5)
                : [ka] "v"(ka), [va] "v"(va) : "memory");
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], 0\n\tds_read_b128 %[n], %[p] offset:1536"
                         : [c] "+v"(Sn0), [n] "=&v"(t6) : [a] "v"(t0), [b] "v"(Qf[0]), [p] "v"(ka) : "memory");
            float mxa = fmaxf(fmaxf(SC(0), SC(1)), SC(2)), mxb = fmaxf(fmaxf(SC(3), SC(4)), SC(5));
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], 0\n\tds_read_b128 %[n], %[p] offset:9728"
                         : [c] "+v"(Sn1), [n] "=&v"(t7) : [a] "v"(t1), [b] "v"(Qf[0]), [p] "v"(ka) : "memory");
            mxa = fmaxf(fmaxf(mxa, SC(6)), SC(7)); mxb = fmaxf(fmaxf(mxb, SC(8)), SC(9)); mxa = fmaxf(fmaxf(mxa, SC(10)), SC(11));
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:2048"
                         : [c] "+v"(Sn0), [n] "+v"(t0) : [a] "v"(t2), [b] "v"(Qf[1]), [p] "v"(ka) : "memory");
            mxa = fmaxf(fmaxf(mxa, SC(12)), SC(13)); mxb = fmaxf(fmaxf(mxb, SC(14)), SC(15)); mxa = fmaxf(fmaxf(mxa, SC(16)), SC(17));
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:10240"
                         : [c] "+v"(Sn1), [n] "+v"(t1) : [a] "v"(t3), [b] "v"(Qf[1]), [p] "v"(ka) : "memory");
            mxa = fmaxf(fmaxf(mxa, SC(18)), SC(19)); mxb = fmaxf(fmaxf(mxb, SC(20)), SC(21)); mxa = fmaxf(fmaxf(mxa, SC(22)), SC(23));
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:2560"
                         : [c] "+v"(Sn0), [n] "+v"(t2) : [a] "v"(t4), [b] "v"(Qf[2]), [p] "v"(ka) : "memory");
            mxa = fmaxf(fmaxf(mxa, SC(24)), SC(25)); mxb = fmaxf(fmaxf(mxb, SC(26)), SC(27)); mxa = fmaxf(fmaxf(mxa, SC(28)), SC(29));
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:10752"
                         : [c] "+v"(Sn1), [n] "+v"(t3) : [a] "v"(t5), [b] "v"(Qf[2]), [p] "v"(ka) : "memory");
            mxb = fmaxf(fmaxf(mxb, SC(30)), SC(31));
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:3072"
                         : [c] "+v"(Sn0), [n] "+v"(t4) : [a] "v"(t6), [b] "v"(Qf[3]), [p] "v"(ka) : "memory");
            float mx = fmaxf(mxa, mxb);
            {   // lanes l and l + 32 hold the two key halves of one query row
                const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
            }
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:11264"
                         : [c] "+v"(Sn1), [n] "+v"(t5) : [a] "v"(t7), [b] "v"(Qf[3]), [p] "v"(ka) : "memory");
            RAISE_CHECK(mx);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:3584"
                         : [c] "+v"(Sn0), [n] "+v"(t6) : [a] "v"(t0), [b] "v"(Qf[4]), [p] "v"(ka) : "memory");
            SOFTMAX_PAIR(0);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:11776"
                         : [c] "+v"(Sn1), [n] "+v"(t7) : [a] "v"(t1), [b] "v"(Qf[4]), [p] "v"(ka) : "memory");
            SOFTMAX_PAIR(1);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:0"
                         : [c] "+v"(Sn0), [n] "+v"(t0) : [a] "v"(t2), [b] "v"(Qf[5]), [p] "v"(va) : "memory");
            SOFTMAX_PAIR(2);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:512"
                         : [c] "+v"(Sn1), [n] "+v"(t1) : [a] "v"(t3), [b] "v"(Qf[5]), [p] "v"(va) : "memory");
            SOFTMAX_PAIR(3);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:1024"
                         : [c] "+v"(Sn0), [n] "+v"(t2) : [a] "v"(t4), [b] "v"(Qf[6]), [p] "v"(va) : "memory");
            SOFTMAX_PAIR(4);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:1536"
                         : [c] "+v"(Sn1), [n] "+v"(t3) : [a] "v"(t5), [b] "v"(Qf[6]), [p] "v"(va) : "memory");
            SOFTMAX_PAIR(5);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:4096"
                         : [c] "+v"(Sn0), [n] "+v"(t4) : [a] "v"(t6), [b] "v"(Qf[7]), [p] "v"(va) : "memory");
            SOFTMAX_PAIR(6);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:4608"
                         : [c] "+v"(Sn1), [n] "+v"(t5) : [a] "v"(t7), [b] "v"(Qf[7]), [p] "v"(va) : "memory");
            SOFTMAX_PAIR(7);
            __builtin_amdgcn_sched_barrier(0);
            const bf16x8 P0 = __builtin_bit_cast(bf16x8, make_uint4(Pk[0], Pk[1], Pk[2], Pk[3]));
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:5120"
                         : [c] "+v"(O[0]), [n] "+v"(t6) : [a] "v"(t0), [b] "v"(P0), [p] "v"(va) : "memory");
            SOFTMAX_PAIR(8);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:5632"
                         : [c] "+v"(O[1]), [n] "+v"(t7) : [a] "v"(t1), [b] "v"(P0), [p] "v"(va) : "memory");
            SOFTMAX_PAIR(9);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:8192"
                         : [c] "+v"(O[2]), [n] "+v"(t0) : [a] "v"(t2), [b] "v"(P0), [p] "v"(va) : "memory");
            SOFTMAX_PAIR(10);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:8704"
                         : [c] "+v"(O[3]), [n] "+v"(t1) : [a] "v"(t3), [b] "v"(P0), [p] "v"(va) : "memory");
            SOFTMAX_PAIR(11);
            __builtin_amdgcn_sched_barrier(0);
            const bf16x8 P1 = __builtin_bit_cast(bf16x8, make_uint4(Pk[4], Pk[5], Pk[6], Pk[7]));
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:9216"
                         : [c] "+v"(O[0]), [n] "+v"(t2) : [a] "v"(t4), [b] "v"(P1), [p] "v"(va) : "memory");
            SOFTMAX_PAIR(12);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:9728"
                         : [c] "+v"(O[1]), [n] "+v"(t3) : [a] "v"(t5), [b] "v"(P1), [p] "v"(va) : "memory");
            SOFTMAX_PAIR(13);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:12288"
                         : [c] "+v"(O[2]), [n] "+v"(t4) : [a] "v"(t6), [b] "v"(P1), [p] "v"(va) : "memory");
            SOFTMAX_PAIR(14);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:12800"
                         : [c] "+v"(O[3]), [n] "+v"(t5) : [a] "v"(t7), [b] "v"(P1), [p] "v"(va) : "memory");
            SOFTMAX_PAIR(15);
            __builtin_amdgcn_sched_barrier(0);
            const bf16x8 P2 = __builtin_bit_cast(bf16x8, make_uint4(Pk[8], Pk[9], Pk[10], Pk[11]));
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:13312"
                         : [c] "+v"(O[0]), [n] "+v"(t6) : [a] "v"(t0), [b] "v"(P2), [p] "v"(va) : "memory");
            l_run += psum;
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]\n\tds_read_b128 %[n], %[p] offset:13824"
                         : [c] "+v"(O[1]), [n] "+v"(t7) : [a] "v"(t1), [b] "v"(P2), [p] "v"(va) : "memory");
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(5)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]"
                         : [c] "+v"(O[2]) : [a] "v"(t2), [b] "v"(P2) : "memory");
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(4)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]"
                         : [c] "+v"(O[3]) : [a] "v"(t3), [b] "v"(P2) : "memory");
            __builtin_amdgcn_sched_barrier(0);
            const bf16x8 P3 = __builtin_bit_cast(bf16x8, make_uint4(Pk[12], Pk[13], Pk[14], Pk[15]));
            asm volatile("s_waitcnt lgkmcnt(3)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]"
                         : [c] "+v"(O[0]) : [a] "v"(t4), [b] "v"(P3) : "memory");
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(2)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]"
                         : [c] "+v"(O[1]) : [a] "v"(t5), [b] "v"(P3) : "memory");
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(1)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]"
                         : [c] "+v"(O[2]) : [a] "v"(t6), [b] "v"(P3) : "memory");
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(0)\n\tv_mfma_f32_32x32x16_bf16 %[c], %[a], %[b], %[c]"
                         : [c] "+v"(O[3]) : [a] "v"(t7), [b] "v"(P3) : "memory");
            __builtin_amdgcn_sched_barrier(0);
            // the operand registers stay reserved until the last matrix instructions have read them
            asm volatile("" : "+v"(t0), "+v"(t1), "+v"(t2), "+v"(t3), "+v"(t4), "+v"(t5), "+v"(t6), "+v"(t7));
// ---- end of generated chunks ----
        }
    };
    // scores of the first tile: the 16 matrix instructions alone
    auto first_scores = [&](f32x16 &Sn0, f32x16 &Sn1, int T) {
        const uint8_t *kt = kring + (T % kNS) * kTile + k_rd;
#pragma unroll
        for (int i = 0; i < 16; ++i) { Sn0[i] = 0.f; Sn1[i] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const bf16x8 k0 = *reinterpret_cast<const bf16x8 *>(kt + ks * 512);
            const bf16x8 k1 = *reinterpret_cast<const bf16x8 *>(kt + 2 * kBlock + ks * 512);
            Sn0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, Qf[ks], Sn0, 0, 0, 0);
            Sn1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, Qf[ks], Sn1, 0, 0, 0);
        }
    };

    // ---- prologue: K four tiles ahead, V three; the first scores wait only for K of the first tile ---------------------
    const bool long_item = t_begin + 3 < n_tiles;
    issue_tile(k_base, kring0, t_begin);
    issue_tile(v_base, vring0, t_begin);
    if (t_begin + 1 < n_tiles) { issue_tile(k_base, kring0, t_begin + 1); issue_tile(v_base, vring0, t_begin + 1); }
    if (t_begin + 2 < n_tiles) { issue_tile(k_base, kring0, t_begin + 2); issue_tile(v_base, vring0, t_begin + 2); }
    if (t_begin + 3 < n_tiles) issue_tile(k_base, kring0, t_begin + 3);
    // the query row, rotated; the softmax scale and log2(e) are folded in before it is rounded to bf16.  Loaded
    // after the first K/V tiles have been requested, so that the two latencies overlap.
    {
        const uint16_t *qrow = a.q + ((int64_t)(q0 + j) * a.n_q_heads + head) * kD;
#pragma unroll
        for (int ks = 0; ks < KSTEPS / 2; ++ks) {
            const int piece = 2 * ks + half;
            uint4 x = *reinterpret_cast<const uint4 *>(qrow + 8 * piece);
            uint4 y = *reinterpret_cast<const uint4 *>(qrow + HALF + 8 * piece);
            float2 cs[8];
            load_cs<STYLE>(a.rope, qpos, piece, cs);
            uint32_t *px = reinterpret_cast<uint32_t *>(&x), *py = reinterpret_cast<uint32_t *>(&y);
#pragma unroll
            for (int w = 0; w < 4; ++w) rotate_dword<STYLE>(px[w], py[w], cs, w, cscale);
            Qf[ks] = __builtin_bit_cast(bf16x8, x);
            Qf[ks + KSTEPS / 2] = __builtin_bit_cast(bf16x8, y);
        }
    }

    if (long_item) { CA_WAIT_VMCNT(12); } else { CA_WAIT_VMCNT(0); }
    __syncthreads();
    first_scores(Sa0, Sa1, t_begin);

    // ---- the walk: per tile one wait + barrier (K(T+1) and V(T) of every wavefront have landed, the slots read a tile
    // ago are free), the refill of those slots, and the pipelined tile.  Two tiles per trip, so that the two score
    // buffers swap roles without a copy.  The last tile multiplies scores of a tile that does not exist (unused).
    auto top = [&](int T) {
        if (T + 3 < n_tiles) { CA_WAIT_VMCNT(8); } else { CA_WAIT_VMCNT(0); }
        __syncthreads();
        if (T + 4 < n_tiles) issue_tile(k_base, kring0, T + 4);
        if (T + 3 < n_tiles) issue_tile(v_base, vring0, T + 3);
    };
    for (int T = t_begin; T < n_tiles; T += 2) {
        top(T);
        tile_block(Sa0, Sa1, Sb0, Sb1, T, T >= w_full);
        if (T + 1 >= n_tiles) break;
        top(T + 1);
        tile_block(Sb0, Sb1, Sa0, Sa1, T + 1, T + 1 >= w_full);
    }
    asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");   // the accumulators written by the last matrix instructions are read below

    // ---- epilogue: normalise and store ------------------------------------------------------------------------------------
    const float l_all = l_run + __shfl_xor(l_run, 32);
    if (item.part >= 0) {
        // keys split over several workgroups: leave the unnormalised sums, the reference maximum and the
        // denominator of this share; combine_kernel merges the shares.  The reference goes out in the units of the
        // other kernels (raw score, before the softmax scale); a row that saw no key of the share reports -inf.
        if (row_valid) {
            const int rt = r - item.row0;
            float *base = a.partial + (int64_t)item.part * a.tile_rows * (kD + 2);
            float *prow = base + (int64_t)rt * kD;
#pragma unroll
            for (int db = 0; db < DBLKS; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const int d = 32 * db + i4 * 8 + half * 4;
                    *reinterpret_cast<float4 *>(prow + d) = make_float4(O[db][4 * i4], O[db][4 * i4 + 1], O[db][4 * i4 + 2], O[db][4 * i4 + 3]);
                }
            if (half == 0) {
                base[(int64_t)a.tile_rows * kD + rt] = seen ? M / cscale : -INFINITY;
                base[(int64_t)a.tile_rows * (kD + 1) + rt] = l_all;
            }
        }
        return;
    }
    if (row_valid) {
        const float inv = 1.f / l_all;
        uint16_t *orow = a.out + ((int64_t)(q0 + j) * a.n_q_heads + head) * kD;
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
#undef SC
#undef RAISE_CHECK
#undef SOFTMAX_PAIR

}  // namespace

hipError_t launch_attn_pp(const AttnArgs &a, hipStream_t stream) {
    if (a.n_items <= 0) return hipSuccess;
    if (a.head_dim != kD || a.tile_rows != 256 || !a.k_rot || !a.v_t || !a.dense_page0 || !a.rot_src_page || !a.rot_pos0 ||
        !a.rot_nvalid || a.n_dense_pages <= 0)
        return hipErrorInvalidValue;
    if (a.n_combine > 0 && (a.partial == nullptr || a.combine == nullptr)) return hipErrorInvalidValue;
    const dim3 rgrid((uint32_t)((a.n_dense_pages + 7) / 8) * 8u * (uint32_t)a.n_kv_heads), grid(a.n_items);
    if (a.rope_style == 0) {
        hipLaunchKernelGGL((prepare_kv_kernel<0>), rgrid, dim3(256), 0, stream, a);
        hipLaunchKernelGGL((attn_pp_kernel<0>), grid, dim3(64 * kNW), 0, stream, a);
    } else {
        hipLaunchKernelGGL((prepare_kv_kernel<1>), rgrid, dim3(256), 0, stream, a);
        hipLaunchKernelGGL((attn_pp_kernel<1>), grid, dim3(64 * kNW), 0, stream, a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.n_combine <= 0) return e;
    return launch_attn_combine(a, stream);
}

}  // namespace ca
