// Measured ceilings printed by the benchmark next to the published peaks (libukst_bench.so; not
// part of the transpose convolution).
// Matrix pipes: a register-resident loop of independent MFMAs, no memory traffic at all.  What it
// reaches is the rate the chip sustains at the clock its power management settles on under matrix
// load; a real kernel cannot beat it.
// Memory: a streaming kernel that reads R bytes and writes W bytes, the traffic of a layer with
// that much input and output.
#include "../../../include/ukst_bench.h"
#include <hip/hip_runtime.h>
#include <stdint.h>

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

// Thread t of the grid reads the 16-byte pieces t, t + T, t + 2T, ... of src (T = threads of the
// grid) and then writes the pieces t, t + T, ... of dst: the launch reads all of src once and
// writes all of dst once, a wave's accesses are consecutive.
__global__ __launch_bounds__(256) void ukst_stream_ceiling_kernel(const uint4* __restrict__ src,
                                                                 size_t nread, uint4* __restrict__ dst,
                                                                 size_t nwrite)
{
    const size_t T = (size_t)gridDim.x * 256, t = (size_t)blockIdx.x * 256 + threadIdx.x;
    uint4 acc = make_uint4(0u, 0u, 0u, 0u);
    for (size_t i = t; i < nread; i += T) {
        const uint4 v = src[i];
        acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
    }
    for (size_t i = t; i < nwrite; i += T) dst[i] = acc;
}

}  // namespace

extern "C" int ukst_bench_stream_ceiling(const void* src, size_t read_bytes, void* dst,
                                         size_t write_bytes, void* stream)
{
    if (!src || !dst || (read_bytes & 15) || (write_bytes & 15) || (((uintptr_t)src | (uintptr_t)dst) & 15))
        return -1;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return -1;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return -1;
    // 8 blocks per compute unit: every SIMD holds two waves per block slot, pieces are strided so
    // that a wave's accesses are consecutive
    hipLaunchKernelGGL(ukst_stream_ceiling_kernel, dim3(8 * cus), dim3(256), 0, (hipStream_t)stream,
                       (const uint4*)src, read_bytes / 16, (uint4*)dst, write_bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

extern "C" double ukst_bench_mfma_ceiling(int dtype, int iters, void* sink, void* stream)
{
    constexpr int UKST_F32 = 0, UKST_BF16_F32 = 1;
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
