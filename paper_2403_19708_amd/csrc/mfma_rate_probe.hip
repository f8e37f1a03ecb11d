// Measurement aid, not part of the library: the bf16 matrix-core rate this GPU sustains when a kernel does nothing but
// issue v_mfma_f32_32x32x16_bf16 back to back (four independent accumulators per wavefront), once with all-zero
// operands and once with operands of random sign, exponent and mantissa.  The published peak (2.5 PFLOP/s) assumes the
// nominal clock; the card lowers its clock under load, and by how much depends on how many bits of the operands
// toggle, so the second figure is the ceiling a kernel working on real data can approach.  Prints one JSON line.
#include <hip/hip_runtime.h>

#include <cstdio>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ inline unsigned mix(unsigned x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

template <bool RANDOM>
__global__ __launch_bounds__(512, 1) void rate_kernel(float *out, int iters) {
    f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    bf16x8 a[4], b[4];
    for (int s = 0; s < 4; ++s)
        for (int e = 0; e < 8; ++e) {
            float va = 0.f, vb = 0.f;
            if (RANDOM) {
                const unsigned h = mix(threadIdx.x * 131u + e * 17u + s * 7919u + blockIdx.x * 104729u);
                va = ((int)(h & 0xffff) - 32768) / 16384.0f;
                vb = ((int)(h >> 16) - 32768) / 16384.0f;
            }
            a[s][e] = (__bf16)va;
            b[s][e] = (__bf16)vb;
        }
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[1], c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2], b[2], c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[3], b[3], c3, 0, 0, 0);
    }
    out[blockIdx.x * 512 + threadIdx.x] = c0[0] + c1[1] + c2[2] + c3[3];
}

template <bool RANDOM>
static double tflops(float *out, int n_cu) {
    const int iters = 20000;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1.0;
    hipLaunchKernelGGL((rate_kernel<RANDOM>), dim3(n_cu), dim3(512), 0, 0, out, iters);     // warm-up
    if (hipDeviceSynchronize() != hipSuccess) return -1.0;
    hipEventRecord(e0);
    hipLaunchKernelGGL((rate_kernel<RANDOM>), dim3(n_cu), dim3(512), 0, 0, out, iters);
    hipEventRecord(e1);
    if (hipEventSynchronize(e1) != hipSuccess) return -1.0;
    float ms = 0.f;
    hipEventElapsedTime(&ms, e0, e1);
    const double flop = (double)n_cu * 8 * iters * 4 * 2.0 * 32 * 32 * 16;
    return flop / (ms * 1e-3) / 1e12;
}

int main() {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, 0) != hipSuccess) { fprintf(stderr, "mfma_rate_probe: no device\n"); return 1; }
    const int n_cu = prop.multiProcessorCount;
    float *out = nullptr;
    if (hipMalloc(&out, (size_t)n_cu * 512 * sizeof(float)) != hipSuccess) { fprintf(stderr, "mfma_rate_probe: hipMalloc failed\n"); return 1; }
    const double z = tflops<false>(out, n_cu), r = tflops<true>(out, n_cu);
    hipFree(out);
    if (z < 0 || r < 0) { fprintf(stderr, "mfma_rate_probe: a launch failed\n"); return 1; }
    printf("{\"compute_units\": %d, \"zero_operands_tflops\": %.1f, \"random_operands_tflops\": %.1f}\n", n_cu, z, r);
    return 0;
}
