// Narrow-channel path (fp32, Cin <= 4, Cout <= 4): memory-bound shapes such as 224x224x3 images.
//
// One lane owns a block of 2 x QH output quads, i.e. 4 consecutive output columns by 2*QH rows,
// for every output channel.  All four parity classes of Algorithm 2 are computed from one
// (QH + ceil(n/2) - 1) x (2 + ceil(n/2) - 1) input window held in registers, so every input pixel
// is fetched once per lane and every kernel tap is used exactly once per quad (Sec. 3.1).
// Everything the lane needs is requested up front (one memory round trip), then each output
// channel is accumulated and written with one 16-byte store per row and lane: a wave writes 1 KiB
// of consecutive floats per store whatever the row pitch.
//
// Edge handling is done by the buffer addressing hardware instead of predicates: each input row
// and each output row gets its own buffer descriptor whose size is exactly that row (or zero if
// the row does not exist).  Out-of-range loads return 0 -- that is the floor(P/2) zero padding of
// Sec. 3.4 -- and out-of-range stores are dropped per dword, so odd output widths and heights
// produce no extra elements.
#include "ukst_internal.h"

namespace ukst {
namespace {

typedef unsigned u2v __attribute__((ext_vector_type(2)));
typedef unsigned u4v __attribute__((ext_vector_type(4)));

constexpr int kRsrcFlags = 0x00020000;  // raw 32-bit buffer, gfx9 family

__device__ __forceinline__ int xcd_contiguous(int bid, int nb)
{
    constexpr int X = 8;
    const int xcd = bid % X, idx = bid / X;
    const int fl = nb / X, rem = nb % X;
    return xcd * fl + (xcd < rem ? xcd : rem) + idx;
}

__device__ __forceinline__ unsigned fbits(float f) { return __builtin_bit_cast(unsigned, f); }

template <int N, int CI, int CO, int QH>
__global__ __launch_bounds__(256) void ukst_narrow_kernel(const float* __restrict__ x,
                                                         const float* __restrict__ w,
                                                         float* __restrict__ y, Geom g,
                                                         int strips, int bands, int nwork)
{
    constexpr int HI = (N + 1) / 2;     // window side of one quad, ceil(n/2)
    constexpr int QW = 2;               // quads per lane along a row
    constexpr int WR = QH + HI - 1;     // window rows held per lane
    constexpr int WC = QW + HI - 1;     // window cols held per lane
    constexpr int NN = N * N;
    constexpr int NNP = (NN + 3) & ~3;  // taps of one (co, ci) pair, padded for 16-byte LDS reads
    __shared__ __align__(16) float wl[CO * CI * NNP];

    const int tid = threadIdx.x;
    for (int e = tid; e < CO * CI * NNP; e += 256) {
        const int pair = e / NNP, t = e - pair * NNP;
        wl[e] = (t < NN) ? w[pair * NN + t] : 0.f;
    }
    __syncthreads();

    // the wave index is uniform by construction; say so, so that row arithmetic stays scalar
    int wid = xcd_contiguous(blockIdx.x, gridDim.x) * 4 + __builtin_amdgcn_readfirstlane(tid >> 6);
    if (wid >= nwork) return;
    const int lane = tid & 63;
    const int strip = wid % strips; wid /= strips;
    const int band = wid % bands;
    const int b = wid / bands;

    const int H = g.H, W = g.W, P = g.P, OH = g.OH, OW = g.OW;
    const int m0 = g.m_min + strip * (64 * QW) + QW * lane;  // first quad column of this lane
    const int k0 = g.k_min + band * QH;                      // first quad row of this wave
    const int j0 = m0 - P, i0 = k0 - P;                      // first input col / row of the window

    // byte offsets of the window columns inside an input row; columns left of the map get an
    // offset that is out of range for any row
    unsigned voff[WC];
#pragma unroll
    for (int v = 0; v < WC; ++v) voff[v] = (j0 + v >= 0) ? (unsigned)(j0 + v) * 4u : 0x80000000u;

    const float* xb = x + (size_t)b * CI * H * W;
    float win[WR][WC][CI];
#pragma unroll
    for (int u = 0; u < WR; ++u) {
        const int i = i0 + u;
        const bool rowok = i >= 0 && i < H;  // wave-uniform
        const int ic = rowok ? i : 0;
#pragma unroll
        for (int ci = 0; ci < CI; ++ci) {
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                (void*)(xb + ((size_t)ci * H + ic) * W), 0, rowok ? W * 4 : 0, kRsrcFlags);
#pragma unroll
            for (int v = 0; v < WC; ++v)
                win[u][v][ci] = __builtin_bit_cast(
                    float, __builtin_amdgcn_raw_buffer_load_b32(rs, voff[v], 0, 0));
        }
    }

    const int ox_first = 2 * m0 - 1 - P;  // class s = 1 column of the lane's first quad; may be -1
    float* yb = y + (size_t)b * CO * OH * OW;

#pragma unroll
    for (int co = 0; co < CO; ++co) {
        float acc[QH][QW][2][2];
#pragma unroll
        for (int qy = 0; qy < QH; ++qy)
#pragma unroll
            for (int qx = 0; qx < QW; ++qx)
                acc[qy][qx][0][0] = acc[qy][qx][0][1] = acc[qy][qx][1][0] = acc[qy][qx][1][1] = 0.f;

#pragma unroll
        for (int ci = 0; ci < CI; ++ci) {
            float wv[NNP];
#pragma unroll
            for (int t = 0; t < NNP; t += 4) {
                const float4 q = *reinterpret_cast<const float4*>(&wl[(co * CI + ci) * NNP + t]);
                wv[t] = q.x; wv[t + 1] = q.y; wv[t + 2] = q.z; wv[t + 3] = q.w;
            }
            // tap (a, t) belongs to class (a & 1, t & 1) and meets window pixel (a/2, t/2)
#pragma unroll
            for (int qy = 0; qy < QH; ++qy)
#pragma unroll
                for (int qx = 0; qx < QW; ++qx)
#pragma unroll
                    for (int a = 0; a < N; ++a)
#pragma unroll
                        for (int t = 0; t < N; ++t)
                            acc[qy][qx][a & 1][t & 1] =
                                fmaf(win[qy + (a >> 1)][qx + (t >> 1)][ci], wv[a * N + t],
                                     acc[qy][qx][a & 1][t & 1]);
        }

#pragma unroll
        for (int qy = 0; qy < QH; ++qy)
#pragma unroll
            for (int r = 1; r >= 0; --r) {
                const int oy = 2 * (k0 + qy) - P - r;  // row class r of quad row k0 + qy
                const bool rowok = oy >= 0 && oy < OH;  // wave-uniform
                const int oyc = rowok ? oy : 0;
                const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                    (void*)(yb + ((size_t)co * OH + oyc) * OW), 0, rowok ? OW * 4 : 0, kRsrcFlags);
                // columns ox_first .. ox_first+3 = classes s = 1, 0, 1, 0
                if (ox_first >= 0) {
                    u4v d;
                    d.x = fbits(acc[qy][0][r][1]); d.y = fbits(acc[qy][0][r][0]);
                    d.z = fbits(acc[qy][1][r][1]); d.w = fbits(acc[qy][1][r][0]);
                    __builtin_amdgcn_raw_buffer_store_b128(d, rs, (unsigned)ox_first * 4u, 0, 0);
                } else {  // first lane of an even-P row: column -1 does not exist
                    u2v d;
                    d.x = fbits(acc[qy][1][r][1]); d.y = fbits(acc[qy][1][r][0]);
                    __builtin_amdgcn_raw_buffer_store_b32(fbits(acc[qy][0][r][0]), rs, 0u, 0, 0);
                    __builtin_amdgcn_raw_buffer_store_b64(d, rs, 4u, 0, 0);
                }
            }
    }
}

template <int N, int CI, int CO, int QH>
hipError_t launch_q(const Geom& g, const float* x, const float* w, float* y, hipStream_t stream)
{
    const int strips = (g.KW + 127) / 128;
    const int bands = (g.KH + QH - 1) / QH;
    const long long nwork = (long long)strips * bands * g.B;
    if (nwork > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((ukst_narrow_kernel<N, CI, CO, QH>), dim3((unsigned)((nwork + 3) / 4)),
                       dim3(256), 0, stream, x, w, y, g, strips, bands, (int)nwork);
    return hipGetLastError();
}

template <int N, int CI, int CO>
hipError_t launch_t(const Geom& g, const float* x, const float* w, float* y, hipStream_t stream)
{
    // Taller lane blocks re-read fewer halo rows and measured faster on HBM-cold data, as long as
    // there are still enough waves to cover the chip (256 CUs x 4 SIMDs).
    const long long waves4 = (long long)((g.KW + 127) / 128) * ((g.KH + 3) / 4) * g.B;
    if (waves4 >= 1024) return launch_q<N, CI, CO, 4>(g, x, w, y, stream);
    return launch_q<N, CI, CO, 2>(g, x, w, y, stream);
}

template <int N, int CI>
hipError_t launch_co(const Geom& g, const float* x, const float* w, float* y, hipStream_t st)
{
    switch (g.Cout) {
        case 1: return launch_t<N, CI, 1>(g, x, w, y, st);
        case 2: return launch_t<N, CI, 2>(g, x, w, y, st);
        case 3: return launch_t<N, CI, 3>(g, x, w, y, st);
        case 4: return launch_t<N, CI, 4>(g, x, w, y, st);
        default: return hipErrorInvalidValue;
    }
}

template <int N>
hipError_t launch_ci(const Geom& g, const float* x, const float* w, float* y, hipStream_t st)
{
    switch (g.Cin) {
        case 1: return launch_co<N, 1>(g, x, w, y, st);
        case 2: return launch_co<N, 2>(g, x, w, y, st);
        case 3: return launch_co<N, 3>(g, x, w, y, st);
        case 4: return launch_co<N, 4>(g, x, w, y, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool narrow_supported(const Geom& g, int dtype)
{
    // buffer offsets are 32-bit byte offsets inside one row
    return dtype == 0 && g.Cin <= 4 && g.Cout <= 4 && g.n <= 5 && g.W < (1 << 28) &&
           g.OW < (1 << 28);
}

hipError_t launch_narrow(const Geom& g, const void* x, const void* w, float* y, hipStream_t stream)
{
    const float* xf = (const float*)x;
    const float* wf = (const float*)w;
    switch (g.n) {
        case 1: return launch_ci<1>(g, xf, wf, y, stream);
        case 2: return launch_ci<2>(g, xf, wf, y, stream);
        case 3: return launch_ci<3>(g, xf, wf, y, stream);
        case 4: return launch_ci<4>(g, xf, wf, y, stream);
        case 5: return launch_ci<5>(g, xf, wf, y, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ukst
