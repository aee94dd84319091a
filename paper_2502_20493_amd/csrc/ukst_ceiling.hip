// Measured ceiling of the matrix pipes, printed by the benchmark next to the published peak: a
// register-resident loop of independent MFMAs, no memory traffic at all.  What it reaches is the
// rate the chip sustains at the clock its power management settles on under matrix load; a real
// kernel cannot beat it.  Not part of the transpose convolution.
#include "../../include/ukst.h"
#include <hip/hip_runtime.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// 4 waves per block, 4 independent accumulator tiles per wave: enough to keep the pipe of every
// SIMD busy without waiting on a result.
template <bool BF16>
__global__ __launch_bounds__(256) void ukst_mfma_ceiling_kernel(float* sink, int iters)
{
    const int lane = threadIdx.x & 63;
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
    // operands with busy bit patterns (data of all zeros would draw less power and clock higher)
    unsigned h = 0x9E3779B9u * (unsigned)(threadIdx.x + 1) + 0x7F4A7C15u * (blockIdx.x + 1);
    float fa[8], fb[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        h = h * 1664525u + 1013904223u;
        fa[e] = ((int)(h >> 8) & 0xFFFF) * (1.f / 65536.f) - 0.5f;
        h = h * 1664525u + 1013904223u;
        fb[e] = ((int)(h >> 8) & 0xFFFF) * (1.f / 65536.f) - 0.5f;
    }
    if constexpr (BF16) {
        bf16x8 a, b;
#pragma unroll
        for (int e = 0; e < 8; ++e) { a[e] = (__bf16)fa[e]; b[e] = (__bf16)fb[e]; }
        for (int i = 0; i < iters; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    } else {
        const float a = fa[0], b = fb[0];
        for (int i = 0; i < iters; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[j][e];
    if (s == 123456.789f) sink[lane] = s;  // keeps the loop alive; practically never taken
}

}  // namespace

extern "C" double ukst_bench_mfma_ceiling(int dtype, int iters, void* sink, void* stream)
{
    if (!sink || iters < 1 || (dtype != UKST_F32 && dtype != UKST_BF16_F32)) return 0.0;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0.0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0.0;
    const int blocks = 2 * cus;
    if (dtype == UKST_BF16_F32)
        hipLaunchKernelGGL(ukst_mfma_ceiling_kernel<true>, dim3(blocks), dim3(256), 0,
                           (hipStream_t)stream, (float*)sink, iters);
    else
        hipLaunchKernelGGL(ukst_mfma_ceiling_kernel<false>, dim3(blocks), dim3(256), 0,
                           (hipStream_t)stream, (float*)sink, iters);
    if (hipGetLastError() != hipSuccess) return 0.0;
    const double per_mfma = dtype == UKST_BF16_F32 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
    return per_mfma * 4.0 * iters * 4.0 * blocks;
}
