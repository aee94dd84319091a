// Direct path: one thread computes one output quad (all four parity classes of Algorithm 2) for a
// small block of output channels.  The input tile plus its halo is staged once in LDS and shared
// by the four classes; kernel taps are wave-uniform and come in through the scalar cache.
#include "ukst_internal.h"

namespace ukst {
namespace {

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
// one rounding to nearest even at the store when the output is bf16
__device__ __forceinline__ void put(float* p, float v) { *p = v; }
__device__ __forceinline__ void put(uint16_t* p, float v) { *p = __builtin_bit_cast(uint16_t, (__bf16)v); }

template <int N, int CO_BLK, int TW, int TH, int CI_CHUNK, typename TIn, typename TOut>
__global__ __launch_bounds__(TW* TH) void ukst_direct_kernel(const TIn* __restrict__ x,
                                                            const TIn* __restrict__ w,
                                                            TOut* __restrict__ y, GeomBase g,
                                                            int tilesX, int tilesY, int coBlocks,
                                                            Epilogue ep)
{
    constexpr int HI = (N + 1) / 2;   // window side = ceil(n/2) (Sec. 3.2)
    constexpr int LR = TH + HI - 1;   // staged rows: tile + halo
    constexpr int LC = TW + HI - 1;   // staged cols
    constexpr int NT = TW * TH;
    __shared__ float tile[CI_CHUNK][LR][LC];

    int bid = xcd_contiguous(blockIdx.x, gridDim.x);
    const int tx = bid % tilesX; bid /= tilesX;
    const int ty = bid % tilesY; bid /= tilesY;
    const int cb = bid % coBlocks;
    const int b = bid / coBlocks;

    const int tid = threadIdx.x;
    const int lx = tid % TW, ly = tid / TW;
    const int k0 = g.k_min + ty * TH, m0 = g.m_min + tx * TW;
    const int i_base = k0 - g.P, j_base = m0 - g.P;  // first input row / col under the tile
    const int co0 = cb * CO_BLK;
    const int H = g.H, W = g.W, Cin = g.Cin;

    float acc[CO_BLK][2][2];
#pragma unroll
    for (int c = 0; c < CO_BLK; ++c) acc[c][0][0] = acc[c][0][1] = acc[c][1][0] = acc[c][1][1] = 0.f;

    const TIn* xb = x + (size_t)b * Cin * H * W;

    for (int ci0 = 0; ci0 < Cin; ci0 += CI_CHUNK) {
        const int nci = (Cin - ci0 < CI_CHUNK) ? Cin - ci0 : CI_CHUNK;
        if (ci0) __syncthreads();
        // stage the tile + halo; out-of-range pixels are the floor(P/2) zero padding of Sec. 3.4
        for (int e = tid; e < nci * (LR * LC); e += NT) {
            const int ci = e / (LR * LC);
            const int rem = e - ci * (LR * LC);
            const int r = rem / LC, c = rem - r * LC;
            const int gi = i_base + r, gj = j_base + c;
            float v = 0.f;
            if (gi >= 0 && gi < H && gj >= 0 && gj < W)
                v = to_f32(xb[((size_t)(ci0 + ci) * H + gi) * W + gj]);
            tile[ci][r][c] = v;
        }
        __syncthreads();

        for (int ci = 0; ci < nci; ++ci) {
            float win[HI][HI];
#pragma unroll
            for (int u = 0; u < HI; ++u)
#pragma unroll
                for (int v = 0; v < HI; ++v) win[u][v] = tile[ci][ly + u][lx + v];
#pragma unroll
            for (int c = 0; c < CO_BLK; ++c) {
                const int co = (co0 + c < g.Cout) ? co0 + c : g.Cout - 1;  // ragged block: clamp
                const TIn* wp = w + ((size_t)co * Cin + (ci0 + ci)) * (N * N);
                // tap (a, t) belongs to class (a & 1, t & 1) and meets window pixel (a/2, t/2)
#pragma unroll
                for (int a = 0; a < N; ++a)
#pragma unroll
                    for (int t = 0; t < N; ++t)
                        acc[c][a & 1][t & 1] =
                            fmaf(win[a >> 1][t >> 1], to_f32(wp[a * N + t]), acc[c][a & 1][t & 1]);
            }
        }
    }

    // store the quad members that exist; odd edges are predicated, nothing extra is written
    const int k = k0 + ly, m = m0 + lx;
    const int oy1 = 2 * k - 1 - g.P, oy0 = oy1 + 1;  // class r = 1 row, class r = 0 row
    const int ox1 = 2 * m - 1 - g.P, ox0 = ox1 + 1;
    const int OH = g.OH, OW = g.OW;
    const bool vy1 = oy1 >= 0 && oy1 < OH, vy0 = oy0 < OH;  // oy0 >= 0 always (k >= k_min)
    const bool vx1 = ox1 >= 0 && ox1 < OW, vx0 = ox0 < OW;
#pragma unroll
    for (int c = 0; c < CO_BLK; ++c) {
        if (co0 + c >= g.Cout) break;
        TOut* yp = y + ((size_t)b * g.Cout + co0 + c) * OH * OW;
        if (has_epilogue(ep)) {  // uniform
            const float bv = ep.bias ? ep.bias[co0 + c] : 0.f;
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int sc = 0; sc < 2; ++sc) acc[c][r][sc] = epilogue(acc[c][r][sc], bv, ep.act);
        }
        if (vy1) {
            TOut* row = yp + (size_t)oy1 * OW;
            if (vx1) put(row + ox1, acc[c][1][1]);
            if (vx0) put(row + ox0, acc[c][1][0]);
        }
        if (vy0) {
            TOut* row = yp + (size_t)oy0 * OW;
            if (vx1) put(row + ox1, acc[c][0][1]);
            if (vx0) put(row + ox0, acc[c][0][0]);
        }
    }
}

template <int N, int CO_BLK, typename TIn, typename TOut>
hipError_t launch_one(const Geom& g, const void* x, const void* w, float* y, hipStream_t stream)
{
    constexpr int TW = 32, TH = 8, CI_CHUNK = 8;
    const int tilesX = (g.KW + TW - 1) / TW, tilesY = (g.KH + TH - 1) / TH;
    const int coBlocks = (g.Cout + CO_BLK - 1) / CO_BLK;
    const long long nb = (long long)tilesX * tilesY * coBlocks * g.B;
    if (nb > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((ukst_direct_kernel<N, CO_BLK, TW, TH, CI_CHUNK, TIn, TOut>), dim3((unsigned)nb),
                       dim3(TW * TH), 0, stream, (const TIn*)x, (const TIn*)w, (TOut*)y, (GeomBase)g, tilesX,
                       tilesY, coBlocks, g.ep);
    return hipGetLastError();
}

template <int N>
hipError_t launch_n(const Geom& g, const void* x, const void* w, float* y, int dtype,
                    hipStream_t stream)
{
    if (dtype == 2) return launch_one<N, 4, uint16_t, uint16_t>(g, x, w, y, stream);
    if (dtype == 1) return launch_one<N, 4, uint16_t, float>(g, x, w, y, stream);
    if (g.Cout == 1) return launch_one<N, 1, float, float>(g, x, w, y, stream);
    if (g.Cout == 3) return launch_one<N, 3, float, float>(g, x, w, y, stream);
    return launch_one<N, 4, float, float>(g, x, w, y, stream);
}

}  // namespace

hipError_t launch_direct(const Geom& g, const void* x, const void* w, float* y, int dtype,
                         hipStream_t stream)
{
    if (narrow_supported(g, dtype)) return launch_narrow(g, x, w, y, stream);
    if (thin_supported(g, dtype)) return launch_thin(g, x, w, y, stream);
    switch (g.n) {
        case 1: return launch_n<1>(g, x, w, y, dtype, stream);
        case 2: return launch_n<2>(g, x, w, y, dtype, stream);
        case 3: return launch_n<3>(g, x, w, y, dtype, stream);
        case 4: return launch_n<4>(g, x, w, y, dtype, stream);
        case 5: return launch_n<5>(g, x, w, y, dtype, stream);
        case 6: return launch_n<6>(g, x, w, y, dtype, stream);
        case 7: return launch_n<7>(g, x, w, y, dtype, stream);
        default: return hipErrorInvalidValue;
    }
}

const char* direct_kernel_name(const Geom& g, int dtype)
{
    return narrow_supported(g, dtype) ? "ukst_narrow_kernel"
           : thin_supported(g, dtype) ? "ukst_thin_kernel" : "ukst_direct_kernel";
}

}  // namespace ukst
