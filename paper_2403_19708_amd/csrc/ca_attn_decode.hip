// Attention of a decode step (Section 3.2.2: one new token per conversation and step; Sections 2.1 and
// 3.4 for what is computed): every (conversation, kv head) has one or two stacked query rows, so the work
// is a matrix-vector product over the whole context and HBM-bound by a wide margin.  It is therefore NOT
// shaped into matrix-core tiles: the keys and values stream from the pages straight into registers with
// fully coalesced 16-byte loads and are consumed by ordinary fp32 arithmetic.
//
//   * One workgroup of 4 wavefronts per work item (a (conversation, kv head) or, when the host split its
//     keys, one share of it).  Wavefront w takes pages first + w, first + w + 4, ...; a page of one head is
//     4 KiB of keys and 4 KiB of values, contiguous.  The loads of the next page are issued before the
//     current one is consumed.
//   * Lane layout: D/8 lanes per key (16 for D = 128, so a load instruction covers 4 keys, a page is 4
//     loads).  For the values a lane owns 8 consecutive head dimensions.  For the keys a lane owns four
//     rotary pairs: with interleaved pairs these are its 8 consecutive dimensions (one 16-byte load), with
//     split-half pairs dimensions 4c..4c+3 and D/2+4c..D/2+4c+3 (two 8-byte loads).
//   * Rotary on load without touching the keys: R(p_q) q . R(t) k = R(p_q - t) q . k, so a lane keeps the
//     query rotated by the relative position of ITS current key (8 floats per row) and advances it by a
//     constant rotation from key to key (4 positions on within a page, 48 + 4 to the wavefront's next
//     page; D = 64: 8 and 48 + 8).  It is re-seeded from the table every 32 pages of a wavefront.
//   * A key's score is the sum over its lanes (four DPP additions inside the 16- or 8-lane group); each lane runs
//     its own online softmax over the keys it has seen (reference maximum, denominator, 8 output sums per
//     row).  At the end the lanes of a wavefront merge by shuffles, the wavefronts through 4 KiB of LDS.
//   * An item that is a share leaves unnormalised sums, maximum and denominator in the partial-result
//     buffer in the layout of the matrix-core kernels; the same combine kernel merges the shares.
//   * Keys and values are read with nontemporal loads: a layer's cache is read once per step and is larger
//     than the last-level cache (measured 58.8 against 63.5 us on 340 MB).
//   * Slots past the end of the context are never dereferenced: their address is clamped to the last
//     visible key (finite data) and their score is masked.
#include "ca_internal.h"

namespace ca {

namespace {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

constexpr int kDecodeWaves = 4;
constexpr int kReseedPages = 32;   // pages a wavefront walks between two seeds of the rotated query

__device__ inline float lo_f(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float hi_f(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ inline uint32_t pack2(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    bf16x2 v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(uint32_t, v);
}

// x + (x of the lane a DPP pattern pairs this lane with); all lanes must be active
template <int CTRL>
__device__ inline float dpp_add(float x) {
    const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true);
    return x + __int_as_float(y);
}
// sum over the aligned group of LPK (8 or 16) lanes, left in every lane of the group: neighbours inside a
// quad, the other pair of the quad, the mirrored lane of the 8-lane half, the mirrored lane of the 16-lane row
template <int LPK>
__device__ inline float group_sum(float x) {
    x = dpp_add<0xB1>(x);      // quad_perm [1,0,3,2]
    x = dpp_add<0x4E>(x);      // quad_perm [2,3,0,1]
    x = dpp_add<0x141>(x);     // row_half_mirror
    if (LPK == 16) x = dpp_add<0x140>(x);   // row_mirror
    return x;
}

struct Softmax {   // one lane's running state for one query row
    float m, l;
    float o[8];
};

__device__ inline void merge(Softmax &a, float m2, float l2, const float (&o2)[8], float cscale) {
    const float M = fmaxf(a.m, m2);
    const float ref = (M == -INFINITY) ? 0.f : M;
    const float wa = __builtin_amdgcn_exp2f((a.m - ref) * cscale);
    const float wb = __builtin_amdgcn_exp2f((m2 - ref) * cscale);
    a.l = a.l * wa + l2 * wb;
#pragma unroll
    for (int i = 0; i < 8; ++i) a.o[i] = a.o[i] * wa + o2[i] * wb;
    a.m = M;
}

// R = stacked query rows handled (1 or 2).  STYLE 0: pairs (i, i + D/2); 1: pairs (2i, 2i + 1).
template <int D, int STYLE, int R>
__global__ __launch_bounds__(64 * kDecodeWaves) void attn_decode_kernel(AttnArgs a) {
    constexpr int HALF = D / 2;
    constexpr int LPK = D / 8;              // lanes per key
    constexpr int KPL = 64 / LPK;           // keys per load instruction
    constexpr int NL = kPageSize / KPL;     // load instructions per page and array
    __shared__ float red[kDecodeWaves][R][D + 2];

    const WorkItem item = a.items[blockIdx.x];
    if (item.seq < 0) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int cl = lane % LPK;              // which 8 dimensions (values) / 4 pairs (keys)
    const int ks = lane / LPK;              // key slot inside a load

    const int c = item.seq;
    const int g = item.kv_head;
    const int G = a.n_q_heads / a.n_kv_heads;
    const int Hkv = a.n_kv_heads;
    const int n = a.n_keep[c];
    const int q0 = a.cu_q[c];
    const int32_t *table = a.block_table + (int64_t)c * a.max_pages;
    const float cscale = a.softmax_scale * 1.4426950408889634f;

    const int row_last = item.row0 + item.n_rows - 1;
    const int kmax = min(n + row_last / G + 1, item.key_end);     // exclusive end of the keys this item reads
    const int first_page = item.key_begin / kPageSize;
    const int last_page = (kmax - 1) / kPageSize;

    // ---- the query rows, unrotated, as the four pairs of this lane ----------------------------------------
    float qx[R][4], qy[R][4];
    int qpos[R], vis_end[R];
    bool row_on[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        row_on[rr] = rr < item.n_rows;
        const int r = item.row0 + (row_on[rr] ? rr : 0);
        const int j = r / G;
        const int head = g * G + (r - j * G);
        qpos[rr] = n + j;
        vis_end[rr] = row_on[rr] ? min(kmax, qpos[rr] + 1) : 0;
        const uint16_t *qrow = a.q + ((int64_t)(q0 + j) * a.n_q_heads + head) * D;
        if (STYLE == 1) {
            const uint4 u = *reinterpret_cast<const uint4 *>(qrow + 8 * cl);
            const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) { qx[rr][k] = lo_f(w[k]); qy[rr][k] = hi_f(w[k]); }
        } else {
            const uint2 ux = *reinterpret_cast<const uint2 *>(qrow + 4 * cl);
            const uint2 uy = *reinterpret_cast<const uint2 *>(qrow + HALF + 4 * cl);
            qx[rr][0] = lo_f(ux.x); qx[rr][1] = hi_f(ux.x); qx[rr][2] = lo_f(ux.y); qx[rr][3] = hi_f(ux.y);
            qy[rr][0] = lo_f(uy.x); qy[rr][1] = hi_f(uy.x); qy[rr][2] = lo_f(uy.y); qy[rr][3] = hi_f(uy.y);
        }
    }
    // constant rotations: KPL positions back (next key of this lane inside a page), and from the last load of
    // a page to the first load of the wavefront's next page (kDecodeWaves pages on, NL - 1 loads back)
    float2 step_in[4], step_page[4];
    {
        const float2 *r1 = a.rope + (int64_t)KPL * HALF + 4 * cl;
        const float2 *r2 = a.rope + (int64_t)(kDecodeWaves * kPageSize - (NL - 1) * KPL) * HALF + 4 * cl;
#pragma unroll
        for (int k = 0; k < 4; ++k) { step_in[k] = r1[k]; step_page[k] = r2[k]; }
    }

    Softmax acc[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        acc[rr].m = -INFINITY;
        acc[rr].l = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[rr].o[i] = 0.f;
    }
    float wx[R][4], wy[R][4];               // the query rotated by (its position - this lane's current key)

    // ---- loads of one page: NL loads of keys (two 8-byte halves for split-half pairs) and NL of values -----
    struct PageRegs {
        u32x4 k[NL];
        u32x4 v[NL];
    };
    auto load_page = [&](int page_idx, PageRegs &p) __attribute__((always_inline)) {
        const int page = table[page_idx];
        const uint16_t *kbase = a.k_pool + ((int64_t)page * Hkv + g) * kPageSize * D;
        const uint16_t *vbase = a.v_pool + ((int64_t)page * Hkv + g) * kPageSize * D;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int t = min(page_idx * kPageSize + i * KPL + ks, kmax - 1);      // clamped: always a visible key
            const int slot = t - page_idx * kPageSize;      // (kmax - 1 lies in the last page, the only one clamped)
            if (STYLE == 1) {
                p.k[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(kbase + slot * D + 8 * cl));
            } else {
                const u32x2 x = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(kbase + slot * D + 4 * cl));
                const u32x2 y = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(kbase + slot * D + HALF + 4 * cl));
                p.k[i] = u32x4{x.x, x.y, y.x, y.y};
            }
            p.v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(vbase + slot * D + 8 * cl));
        }
    };

    auto seed = [&](int t) __attribute__((always_inline)) {
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            const int rel = max(qpos[rr] - t, 0);            // a key past the row's position is masked anyway
            const float2 *row = a.rope + (int64_t)rel * HALF + 4 * cl;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float2 cs = row[k];
                wx[rr][k] = qx[rr][k] * cs.x - qy[rr][k] * cs.y;
                wy[rr][k] = qy[rr][k] * cs.x + qx[rr][k] * cs.y;
            }
        }
    };
    auto advance = [&](const float2 (&st)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int rr = 0; rr < R; ++rr)
#pragma unroll
            for (int k = 0; k < 4; ++k) {              // rotate by minus the step
                const float x = wx[rr][k], y = wy[rr][k];
                wx[rr][k] = x * st[k].x + y * st[k].y;
                wy[rr][k] = y * st[k].x - x * st[k].y;
            }
    };

    auto consume = [&](int page_idx, const PageRegs &p) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int t = page_idx * kPageSize + i * KPL + ks;
            float kx[4], ky[4];
            if (STYLE == 1) {
                const uint32_t w[4] = {p.k[i].x, p.k[i].y, p.k[i].z, p.k[i].w};
#pragma unroll
                for (int k = 0; k < 4; ++k) { kx[k] = lo_f(w[k]); ky[k] = hi_f(w[k]); }
            } else {
                kx[0] = lo_f(p.k[i].x); kx[1] = hi_f(p.k[i].x); kx[2] = lo_f(p.k[i].y); kx[3] = hi_f(p.k[i].y);
                ky[0] = lo_f(p.k[i].z); ky[1] = hi_f(p.k[i].z); ky[2] = lo_f(p.k[i].w); ky[3] = hi_f(p.k[i].w);
            }
            const uint32_t vw[4] = {p.v[i].x, p.v[i].y, p.v[i].z, p.v[i].w};
            float v[8];
#pragma unroll
            for (int k = 0; k < 4; ++k) { v[2 * k] = lo_f(vw[k]); v[2 * k + 1] = hi_f(vw[k]); }
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                float s = 0.f;
#pragma unroll
                for (int k = 0; k < 4; ++k) s += wx[rr][k] * kx[k] + wy[rr][k] * ky[k];
                s = group_sum<LPK>(s);
                s = (t < vis_end[rr]) ? s : -INFINITY;
                const float m_new = fmaxf(acc[rr].m, s);
                const float ref = (m_new == -INFINITY) ? 0.f : m_new;
                const float alpha = __builtin_amdgcn_exp2f((acc[rr].m - ref) * cscale);
                const float pr = __builtin_amdgcn_exp2f((s - ref) * cscale);
                acc[rr].m = m_new;
                acc[rr].l = acc[rr].l * alpha + pr;
#pragma unroll
                for (int d = 0; d < 8; ++d) acc[rr].o[d] = acc[rr].o[d] * alpha + pr * v[d];
            }
            if (i + 1 < NL) advance(step_in);
        }
    };

    // ---- the walk: wavefront w takes pages first_page + w + 4i ------------------------------------------------
    int pg = first_page + wave;
    if (pg <= last_page) {
        PageRegs cur, nxt;
        load_page(pg, cur);
        int since_seed = kReseedPages;
        while (true) {
            const int pg_next = pg + kDecodeWaves;
            const bool more = pg_next <= last_page;
            if (more) load_page(pg_next, nxt);
            if (since_seed == kReseedPages) {
                seed(pg * kPageSize + ks);
                since_seed = 0;
            }
            consume(pg, cur);
            if (!more) break;
            advance(step_page);
            ++since_seed;
            cur = nxt;
            pg = pg_next;
        }
    }

    // ---- merge: the key slots of a wavefront by shuffles, the wavefronts through LDS ---------------------------
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
#pragma unroll
        for (int off = LPK; off < 64; off <<= 1) {
            const float m2 = __shfl_xor(acc[rr].m, off);
            const float l2 = __shfl_xor(acc[rr].l, off);
            float o2[8];
#pragma unroll
            for (int d = 0; d < 8; ++d) o2[d] = __shfl_xor(acc[rr].o[d], off);
            merge(acc[rr], m2, l2, o2, cscale);
        }
        if (ks == 0) {
#pragma unroll
            for (int d = 0; d < 8; ++d) red[wave][rr][8 * cl + d] = acc[rr].o[d];
            if (cl == 0) {
                red[wave][rr][D] = acc[rr].m;
                red[wave][rr][D + 1] = acc[rr].l;
            }
        }
    }
    __syncthreads();
    const int tid = threadIdx.x;
    if (tid >= R * LPK) return;
    const int rr = tid / LPK, cc = tid % LPK;
    if (rr >= item.n_rows) return;
    Softmax tot;
    tot.m = red[0][rr][D];
    tot.l = red[0][rr][D + 1];
#pragma unroll
    for (int d = 0; d < 8; ++d) tot.o[d] = red[0][rr][8 * cc + d];
#pragma unroll
    for (int w = 1; w < kDecodeWaves; ++w) {
        float o2[8];
#pragma unroll
        for (int d = 0; d < 8; ++d) o2[d] = red[w][rr][8 * cc + d];
        merge(tot, red[w][rr][D], red[w][rr][D + 1], o2, cscale);
    }
    if (item.part >= 0) {
        float *base = a.partial + (int64_t)item.part * a.tile_rows * (D + 2);
        float *prow = base + (int64_t)rr * D + 8 * cc;
        *reinterpret_cast<float4 *>(prow) = make_float4(tot.o[0], tot.o[1], tot.o[2], tot.o[3]);
        *reinterpret_cast<float4 *>(prow + 4) = make_float4(tot.o[4], tot.o[5], tot.o[6], tot.o[7]);
        if (cc == 0) {
            base[(int64_t)a.tile_rows * D + rr] = tot.m;
            base[(int64_t)a.tile_rows * (D + 1) + rr] = tot.l;
        }
        return;
    }
    const int r = item.row0 + rr;
    const int j = r / G;
    const int head = g * G + (r - j * G);
    const float inv = 1.f / tot.l;
    uint4 ob;
    ob.x = pack2(tot.o[0] * inv, tot.o[1] * inv);
    ob.y = pack2(tot.o[2] * inv, tot.o[3] * inv);
    ob.z = pack2(tot.o[4] * inv, tot.o[5] * inv);
    ob.w = pack2(tot.o[6] * inv, tot.o[7] * inv);
    *reinterpret_cast<uint4 *>(a.out + ((int64_t)(q0 + j) * a.n_q_heads + head) * D + 8 * cc) = ob;
}

template <int R>
hipError_t launch_rows(const AttnArgs &a, hipStream_t stream) {
    const dim3 grid(a.n_items), block(64 * kDecodeWaves);
    if (a.head_dim == 128 && a.rope_style == 0) hipLaunchKernelGGL((attn_decode_kernel<128, 0, R>), grid, block, 0, stream, a);
    else if (a.head_dim == 128 && a.rope_style == 1) hipLaunchKernelGGL((attn_decode_kernel<128, 1, R>), grid, block, 0, stream, a);
    else if (a.head_dim == 64 && a.rope_style == 0) hipLaunchKernelGGL((attn_decode_kernel<64, 0, R>), grid, block, 0, stream, a);
    else if (a.head_dim == 64 && a.rope_style == 1) hipLaunchKernelGGL((attn_decode_kernel<64, 1, R>), grid, block, 0, stream, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace

// max_rows: the most stacked rows any item of the plan has (1 or 2); every item must start at row 0
hipError_t launch_attn_decode(const AttnArgs &a, int max_rows, hipStream_t stream) {
    if (a.n_items <= 0) return hipSuccess;
    if (max_rows < 1 || max_rows > kAttnDecodeMaxRows) return hipErrorInvalidValue;
    if (a.n_combine > 0 && (a.partial == nullptr || a.combine == nullptr)) return hipErrorInvalidValue;
    const hipError_t e = max_rows == 1 ? launch_rows<1>(a, stream) : launch_rows<2>(a, stream);
    if (e != hipSuccess || a.n_combine <= 0) return e;
    return launch_attn_combine(a, stream);
}

}  // namespace ca
