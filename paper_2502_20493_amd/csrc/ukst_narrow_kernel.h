// Narrow-channel path (fp32, Cin <= 4, Cout <= 4): memory-bound shapes such as 224x224x3 images.
//
// One lane owns 4 consecutive output columns (a 16-byte aligned group counted from column 0) by
// 2*QH output rows, for every output channel.  The four parity classes of Algorithm 2 appear as
// compile-time constants: output column c of the group uses the kernel taps of column parity
// (c + P) & 1 and output row class r the taps of row parity r (Sec. 3.1-3.2), so every tap is used
// exactly once per output it belongs to and no bed-of-nails zero is ever multiplied.  Everything a
// lane needs of the input -- a (QH + ceil(n/2) - 1) row window -- is requested up front (one memory
// round trip), then each output channel is accumulated and written with one 16-byte store per
// row and lane: a wave writes 1 KiB of consecutive floats per store whatever the row pitch.
//
// Edge handling is done by the buffer addressing hardware instead of predicates.  One descriptor
// describes the image of the batch item; for each row its size field is set to the end of that
// row (or to zero if the row does not exist) and the scalar offset to the start of the row, both
// of which take part in the hardware range check.  Loads beyond the right edge or from a missing
// row return 0 -- that is the floor(P/2) zero padding of Sec. 3.4 -- and stores beyond the right
// edge or to a missing row are dropped per dword, so odd output widths and heights produce no
// extra elements.  Columns left of the map get an offset that is out of range for every row.
#pragma once
#include "ukst_internal.h"

namespace ukst {
namespace narrow {

typedef unsigned u2v __attribute__((ext_vector_type(2)));
typedef unsigned u3v __attribute__((ext_vector_type(3)));
typedef unsigned u4v __attribute__((ext_vector_type(4)));

constexpr int kRsrcFlags = 0x00020000;  // raw 32-bit buffer, gfx9 family
constexpr int kFarBand = 0x20000000;         // a quad row whose input and output rows do not exist

__device__ __forceinline__ unsigned fbits(float f) { return __builtin_bit_cast(unsigned, f); }

// EPI: the fused epilogue (bias, activation) is compiled in between the sums and the stores; the
// plain instances keep sums and stores in one block of straight-line code.
template <int N, int CI, int CO, int QH, bool PE, bool EPI>
__global__ __launch_bounds__(256) void ukst_narrow_kernel(const float* __restrict__ x,
                                                         const float* __restrict__ w,
                                                         float* __restrict__ y, GeomBase g,
                                                         int strips, int bands, int nwork,
                                                         Epilogue ep)
{
    constexpr int HI = (N + 1) / 2;  // taps of even parity along one axis, ceil(n/2)
    constexpr int LO = N / 2;        // taps of odd parity, floor(n/2)
    constexpr int WR = QH + HI - 1;  // window rows held per lane
    // PE (P even): the lane's columns have tap parities 0,1,0,1 and their windows start 0,1,1,2
    // input columns right of the lane's first; P odd: parities 1,0,1,0 and starts 0,0,1,1
    constexpr int WC = (PE ? (HI > LO + 1 ? HI : LO + 1) : HI) + 1;  // window cols held per lane
    constexpr int NN = N * N;
    constexpr int NNP = (NN + 3) & ~3;  // taps of one (co, ci) pair, padded for 16-byte LDS reads
    __shared__ __align__(16) float wl[CO * CI * NNP];

    const int tid = threadIdx.x;
    // the wave index is uniform by construction; say so, so that row arithmetic stays scalar
    int wid = xcd_contiguous(blockIdx.x, gridDim.x) * 4 + __builtin_amdgcn_readfirstlane(tid >> 6);
    // a wave past the end of the work list keeps running (it must reach the barrier below) on a
    // band far outside the map: none of its rows exists
    const bool idle = wid >= nwork;
    const int lane = tid & 63;
    const int strip = wid % strips; wid /= strips;
    const int band = wid % bands;
    const int b = idle ? 0 : wid / bands;

    const int H = g.H, W = g.W, P = g.P, OH = g.OH, OW = g.OW;
    const int lg = strip * 64 + lane;  // the lane's column group
    const int j0 = 2 * lg - (P >> 1);  // first input column of the lane's window

    const float* xb = x + (size_t)b * CI * H * W;
    const unsigned xrow = (unsigned)W * 4u, xplane = (unsigned)H * xrow;
    // window of the band whose first quad row is k0: tap row a of output row 2k - P - (a & 1)
    // meets input row k - P + a/2
    // One load fetches the lane's WC consecutive window columns of a row: the address unit takes
    // as long for a 4-byte load as for a 16-byte one, and it is what bounds the read phase of
    // this kernel.  Dwords past the end of the row come back as 0 one by one, but a load whose
    // first byte lies left of the row returns nothing at all: a lane whose window starts left of
    // the map (floor(P/2) > 0) loads from column 0 instead and shifts the
    // result to the right afterwards.
    const int left = j0 < 0 ? (-j0 < WC ? -j0 : WC) : 0;  // window columns left of the map
    const unsigned woff = j0 < 0 ? 0u : (unsigned)j0 * 4u;
    // wave-uniform: lane 0 of the wave has the leftmost window; with floor(P/2) > 128 the waves
    // of later strips start left of the map too
    const bool shifts = 128 * strip < (P >> 1);
    auto load_window = [&](int k0, float (&win)[WR][WC][CI]) {
        const int i0 = k0 - P;
#pragma unroll
        for (int u = 0; u < WR; ++u) {
            const int i = i0 + u;
            const bool rowok = i >= 0 && i < H;  // wave-uniform
#pragma unroll
            for (int ci = 0; ci < CI; ++ci) {
                // (for a missing row the offset is meaningless and the size field is zero)
                const unsigned start = (unsigned)ci * xplane + (unsigned)i * xrow;
                const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                    (void*)xb, 0, rowok ? (int)(start + xrow) : 0, kRsrcFlags);
                unsigned e[WC];  // elements by value: a bit cast of a vector element reads element 0
                if constexpr (WC == 4) {
                    const u4v t = __builtin_amdgcn_raw_buffer_load_b128(rs, woff, start, 0);
                    e[0] = t.x; e[1] = t.y; e[2] = t.z; e[3] = t.w;
                } else if constexpr (WC == 3) {
                    const u3v t = __builtin_amdgcn_raw_buffer_load_b96(rs, woff, start, 0);
                    e[0] = t.x; e[1] = t.y; e[2] = t.z;
                } else if constexpr (WC == 2) {
                    const u2v t = __builtin_amdgcn_raw_buffer_load_b64(rs, woff, start, 0);
                    e[0] = t.x; e[1] = t.y;
                } else {
                    e[0] = __builtin_amdgcn_raw_buffer_load_b32(rs, woff, start, 0);
                }
#pragma unroll
                for (int v = 0; v < WC; ++v) win[u][v][ci] = __uint_as_float(e[v]);
            }
        }
    };
    // moves a freshly loaded window `left` columns to the right, zeros coming in
    auto shift_window = [&](float (&win)[WR][WC][CI]) {
        if (!shifts) return;
#pragma unroll
        for (int s = 1; s <= WC; ++s) {
            if (s > (P >> 1)) break;  // wave-uniform: no lane is further left than floor(P/2)
            const bool m = left >= s;
#pragma unroll
            for (int u = 0; u < WR; ++u)
#pragma unroll
                for (int ci = 0; ci < CI; ++ci) {
#pragma unroll
                    for (int v = WC - 1; v >= 1; --v) win[u][v][ci] = m ? win[u][v - 1][ci] : win[u][v][ci];
                    win[u][0][ci] = m ? 0.f : win[u][0][ci];
                }
        }
    };

    float* yb = y + (size_t)b * CO * OH * OW;
    const unsigned yrow = (unsigned)OW * 4u, yplane = (unsigned)OH * yrow;
    const unsigned ovoff = (unsigned)lg * 16u;  // output columns 4*lg .. 4*lg + 3

    auto emit = [&](int k0, const float (&win)[WR][WC][CI]) {
#pragma unroll
        for (int co = 0; co < CO; ++co) {
            float acc[QH][2][4];
#pragma unroll
            for (int qy = 0; qy < QH; ++qy)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[qy][0][c] = acc[qy][1][c] = 0.f;

#pragma unroll
            for (int ci = 0; ci < CI; ++ci) {
                float wv[NNP];
#pragma unroll
                for (int t = 0; t < NNP; t += 4) {
                    const float4 q = *reinterpret_cast<const float4*>(&wl[(co * CI + ci) * NNP + t]);
                    wv[t] = q.x; wv[t + 1] = q.y; wv[t + 2] = q.z; wv[t + 3] = q.w;
                }
#pragma unroll
                for (int qy = 0; qy < QH; ++qy)
#pragma unroll
                    for (int a = 0; a < N; ++a)
#pragma unroll
                        for (int t = 0; t < N; ++t)
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                const int sc = PE ? (c & 1) : ((c + 1) & 1);   // tap parity of col c
                                const int jr = PE ? ((c + 1) >> 1) : (c >> 1);  // its window start
                                if ((t & 1) == sc)
                                    acc[qy][a & 1][c] = fmaf(win[qy + (a >> 1)][jr + (t >> 1)][ci],
                                                             wv[a * N + t], acc[qy][a & 1][c]);
                            }
            }

            if constexpr (EPI) {
                const float bv = ep.bias ? ep.bias[co] : 0.f;
#pragma unroll
                for (int qy = 0; qy < QH; ++qy)
#pragma unroll
                    for (int r = 0; r < 2; ++r)
#pragma unroll
                        for (int c = 0; c < 4; ++c) acc[qy][r][c] = epilogue(acc[qy][r][c], bv, ep.act);
            }
#pragma unroll
            for (int qy = 0; qy < QH; ++qy)
#pragma unroll
                for (int r = 1; r >= 0; --r) {
                    const int oy = 2 * (k0 + qy) - P - r;   // row class r of quad row k0 + qy
                    const bool rowok = oy >= 0 && oy < OH;  // wave-uniform
                    const unsigned start = (unsigned)co * yplane + (unsigned)oy * yrow;
                    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                        (void*)yb, 0, rowok ? (int)(start + yrow) : 0, kRsrcFlags);
                    u4v d;
                    d.x = fbits(acc[qy][r][0]); d.y = fbits(acc[qy][r][1]);
                    d.z = fbits(acc[qy][r][2]); d.w = fbits(acc[qy][r][3]);
                    // The row offset goes into the vector offset, not the scalar one: a 16-byte
                    // store that takes a scalar offset was seen to pick up the next instruction's
                    // write to its first data register in lanes 12-15 of each 16, and the
                    // compiler only keeps the two apart for stores without a scalar offset.
                    __builtin_amdgcn_raw_buffer_store_b128(d, rs, ovoff + start, 0, 0);
                }
        }
    };

    float win[WR][WC][CI];
    const int k0 = idle ? kFarBand : g.k_min + band * QH;
    load_window(k0, win);
    __builtin_amdgcn_sched_barrier(0);

    // The block's weights are requested behind the window, not before it: vector loads return in
    // order, and every block of the grid asks for these same few cache lines at the same moment,
    // which was measured to be the slowest request of the kernel.
    constexpr int WPT = (CO * CI * NNP + 255) / 256;  // staged weights per thread
    float wstage[WPT];
#pragma unroll
    for (int k = 0; k < WPT; ++k) {
        const int e = tid + 256 * k;
        const int pair = e / NNP, t = e - pair * NNP;
        wstage[k] = (e < CO * CI * NNP && t < NN) ? w[pair * NN + t] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < WPT; ++k) {
        const int e = tid + 256 * k;
        if (e < CO * CI * NNP) wl[e] = wstage[k];
    }
    __syncthreads();

    shift_window(win);
    emit(k0, win);
}

template <int N, int CI, int CO, int QH, bool PE>
hipError_t launch_q(const Geom& g, const float* x, const float* w, float* y, hipStream_t stream)
{
    const int strips = (g.OW + 255) / 256;                  // 64 lanes x 4 output columns
    const int bands = (g.KH + QH - 1) / QH;                 // QH quad rows each
    const long long nwork = (long long)strips * bands * g.B;
    if (nwork > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    // the instances with an epilogue exist for QH = 2 only (see launch_t)
    if constexpr (QH == 2) {
        if (has_epilogue(g.ep)) {
            hipLaunchKernelGGL((ukst_narrow_kernel<N, CI, CO, QH, PE, true>),
                               dim3((unsigned)((nwork + 3) / 4)), dim3(256), 0, stream, x, w, y,
                               (GeomBase)g, strips, bands, (int)nwork, g.ep);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((ukst_narrow_kernel<N, CI, CO, QH, PE, false>), dim3((unsigned)((nwork + 3) / 4)),
                       dim3(256), 0, stream, x, w, y, (GeomBase)g, strips, bands, (int)nwork, g.ep);
    return hipGetLastError();
}

template <int N, int CI, int CO, bool PE>
hipError_t launch_t(const Geom& g, const float* x, const float* w, float* y, hipStream_t stream)
{
    // Taller lane blocks re-read fewer halo rows but mean fewer, heavier waves; measured on
    // 224x224x3 images, 4 quad rows per lane win for n <= 3 and 2 for the larger kernels (whose
    // lanes already carry more multiplications per output), and 4 only pay off while there are
    // still enough waves to cover the chip (256 CUs x 4 SIMDs).
    const long long waves4 = (long long)((g.OW + 255) / 256) * ((g.KH + 3) / 4) * g.B;
    if (N <= 3 && waves4 >= 1024 && !has_epilogue(g.ep)) return launch_q<N, CI, CO, 4, PE>(g, x, w, y, stream);
    return launch_q<N, CI, CO, 2, PE>(g, x, w, y, stream);
}

template <int N, int CI, int CO>
hipError_t launch_p(const Geom& g, const float* x, const float* w, float* y, hipStream_t stream)
{
    return (g.P & 1) ? launch_t<N, CI, CO, false>(g, x, w, y, stream)
                     : launch_t<N, CI, CO, true>(g, x, w, y, stream);
}

template <int N, int CI>
hipError_t launch_co(const Geom& g, const float* x, const float* w, float* y, hipStream_t st)
{
    switch (g.Cout) {
        case 1: return launch_p<N, CI, 1>(g, x, w, y, st);
        case 2: return launch_p<N, CI, 2>(g, x, w, y, st);
        case 3: return launch_p<N, CI, 3>(g, x, w, y, st);
        case 4: return launch_p<N, CI, 4>(g, x, w, y, st);
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

}  // namespace narrow
}  // namespace ukst
