// Scalar fp32 attention kernel: the same operation as the MFMA kernel (Sections 2.1, 3.1, 3.4)
// computed the slow way, one wavefront per (new token, query head), no matrix cores, no
// intermediate rounding.  It exists to check the plumbing (paging, rebased positions, GQA head
// mapping) and the MFMA kernel against a second device implementation; it is not a fast path.
#include "ca_internal.h"

namespace ca {

namespace {

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

__device__ inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int D>
__global__ __launch_bounds__(64) void attn_ref_kernel(AttnArgs a) {
    constexpr int HALF = D / 2;
    const int i = blockIdx.x;   // new token (flat over the batch)
    const int h = blockIdx.y;   // query head
    const int lane = threadIdx.x;
    const int c = a.q_seq[i];
    const int pos = a.q_pos[i];  // = n_keep + j; keys 0..pos are visible
    const int G = a.n_q_heads / a.n_kv_heads;
    const int g = h / G;
    const int32_t *table = a.block_table + (int64_t)c * a.max_pages;

    __shared__ float qr[D];
    {   // rotate the query at its rebased position
        const uint16_t *q = a.q + ((int64_t)i * a.n_q_heads + h) * D;
        for (int p = lane; p < HALF; p += 64) {
            const int ia = a.rope_style == 0 ? p : 2 * p;
            const int ib = a.rope_style == 0 ? p + HALF : 2 * p + 1;
            const float2 cs = a.rope[(int64_t)pos * HALF + p];
            const float x = bf16_to_f32(q[ia]), y = bf16_to_f32(q[ib]);
            qr[ia] = x * cs.x - y * cs.y;
            qr[ib] = y * cs.x + x * cs.y;
        }
    }
    __syncthreads();

    float m = -INFINITY, l = 0.f;
    float o[D];
#pragma unroll
    for (int d = 0; d < D; ++d) o[d] = 0.f;

    for (int t = lane; t <= pos; t += 64) {
        const int page = table[t / kPageSize];
        const int64_t off = (((int64_t)page * a.n_kv_heads + g) * kPageSize + t % kPageSize) * D;
        const uint16_t *k = a.k_pool + off;
        const uint16_t *v = a.v_pool + off;
        float s = 0.f;
        for (int p = 0; p < HALF; ++p) {
            const int ia = a.rope_style == 0 ? p : 2 * p;
            const int ib = a.rope_style == 0 ? p + HALF : 2 * p + 1;
            const float2 cs = a.rope[(int64_t)t * HALF + p];
            const float x = bf16_to_f32(k[ia]), y = bf16_to_f32(k[ib]);
            s += qr[ia] * (x * cs.x - y * cs.y) + qr[ib] * (y * cs.x + x * cs.y);
        }
        s *= a.softmax_scale;
        const float m_new = fmaxf(m, s);
        const float alpha = expf(m - m_new);  // exp(-inf) = 0 on the first key
        const float p = expf(s - m_new);
        l = l * alpha + p;
#pragma unroll
        for (int d = 0; d < D; ++d) o[d] = o[d] * alpha + p * bf16_to_f32(v[d]);
        m = m_new;
    }

    // merge the 64 partial softmaxes
    float m_all = m;
    for (int w = 32; w >= 1; w >>= 1) m_all = fmaxf(m_all, __shfl_xor(m_all, w));
    const float f = (m == -INFINITY) ? 0.f : expf(m - m_all);
    l *= f;
    for (int w = 32; w >= 1; w >>= 1) l += __shfl_xor(l, w);
    uint16_t *out = a.out + ((int64_t)i * a.n_q_heads + h) * D;
#pragma unroll
    for (int d = 0; d < D; ++d) {
        float x = o[d] * f;
        for (int w = 32; w >= 1; w >>= 1) x += __shfl_xor(x, w);
        if (lane == (d & 63)) out[d] = f32_to_bf16_rne(x / l);
    }
}

}  // namespace

hipError_t launch_attn_ref(const AttnArgs &a, hipStream_t stream) {
    if (a.total_q <= 0) return hipSuccess;
    dim3 grid(a.total_q, a.n_q_heads);
    if (a.head_dim == 128)
        hipLaunchKernelGGL(attn_ref_kernel<128>, grid, dim3(64), 0, stream, a);
    else if (a.head_dim == 64)
        hipLaunchKernelGGL(attn_ref_kernel<64>, grid, dim3(64), 0, stream, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ca
