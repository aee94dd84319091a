// The two generalisations Sec. 5 of the paper points to, on the vector ALUs, one kernel for both:
//
//  * transpose convolution with a general stride s: s-1 zeros are inserted between neighbouring
//    pixels (Algorithm 1 with s in place of 2), so tap a of output row oy meets a pixel only where
//    oy + a - P is a multiple of s.  Algorithm 2 carries over with s*s classes instead of four:
//    row class r = (P - oy) mod s, taps r, r+s, r+2s, ... (the sub-kernel k_rc[u][v] =
//    K[r+s*u][c+s*v]), tap r+s*u reads input row (oy + r - P)/s + u.  Each thread selects the
//    class of its output pixel at run time and never touches an inserted zero.
//  * dilated convolution with dilation d: here the KERNEL is the bed of nails (d-1 zeros between
//    neighbouring taps), and the computation pattern is applied to the segregated INPUT: output
//    pixel (oy, ox) only meets input pixels congruent to (oy - P, ox - P) modulo d, i.e. one of the
//    d*d sub-sampled input maps, with the unmodified n x n kernel.  A thread reads its sub-map in
//    place (input row oy - P + d*a for tap a); the sub-maps are never built.
//
// Both are the gather  y[oy][ox] = sum_ci sum_{u<Tr} sum_{v<Tc} x[i0 + u*xs][j0 + v*xs] *
// w[r + u*ws][c + v*ws]  with (xs, ws) = (1, s) or (d, 1).  Block = 32 x 8 output pixels x 8
// output channels; the weights of 8 input channels at a time sit in LDS as [ci][tap][co] and are
// read as two 16-byte broadcasts per input value; out-of-range window pixels (the padding) are
// skipped by a bounds predicate.
#include "ukst_internal.h"

namespace ukst {
namespace {

constexpr int CO_BLK = 8;   // output channels per thread
constexpr int CI_CH = 8;    // input channels per weight stage
constexpr int MAX_NN = 49;  // n <= 7

struct GenArgs {
    int B, Cin, Cout, H, W, n, P, k, OH, OW;
    int dilated;  // 0: stride-k transpose convolution, 1: dilation-k convolution
    int tilesX, tilesY, coBlocks;
};

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(uint16_t v) { return __uint_as_float((unsigned)v << 16); }

template <typename TIn>
__global__ __launch_bounds__(256) void ukst_general_kernel(const TIn* __restrict__ x,
                                                          const TIn* __restrict__ w,
                                                          float* __restrict__ y, GenArgs a)
{
    __shared__ __align__(16) float wl[CI_CH * MAX_NN * CO_BLK];
    const int tid = threadIdx.x;
    int bid = blockIdx.x;
    const int tile = bid % (a.tilesX * a.tilesY); bid /= a.tilesX * a.tilesY;
    const int cob = bid % a.coBlocks;
    const int b = bid / a.coBlocks;
    const int ox = (tile % a.tilesX) * 32 + (tid & 31);
    const int oy = (tile / a.tilesX) * 8 + (tid >> 5);
    const bool valid = ox < a.OW && oy < a.OH;
    const int co0 = cob * CO_BLK;
    const int n = a.n, NN = n * n, k = a.k;

    // run-time class selection: first tap (r, c), tap stride, window start, input stride, taps
    int r = 0, c = 0, i0, j0, Tr, Tc, xstep, wstep;
    if (a.dilated) {
        i0 = oy - a.P; j0 = ox - a.P; Tr = Tc = n; xstep = k; wstep = 1;
    } else {
        r = ((a.P - oy) % k + k) % k;
        c = ((a.P - ox) % k + k) % k;
        i0 = (oy + r - a.P) / k;  // exact: the numerator is a multiple of k (also when negative)
        j0 = (ox + c - a.P) / k;
        Tr = r < n ? (n - r + k - 1) / k : 0;
        Tc = c < n ? (n - c + k - 1) / k : 0;
        xstep = 1; wstep = k;
    }

    float acc[CO_BLK];
#pragma unroll
    for (int co = 0; co < CO_BLK; ++co) acc[co] = 0.f;

    for (int ci0 = 0; ci0 < a.Cin; ci0 += CI_CH) {
        __syncthreads();
        for (int e = tid; e < CI_CH * NN * CO_BLK; e += 256) {
            const int co = e % CO_BLK, t = (e / CO_BLK) % NN, ci = e / (CO_BLK * NN);
            float v = 0.f;
            if (co0 + co < a.Cout && ci0 + ci < a.Cin)
                v = to_f32(w[((size_t)(co0 + co) * a.Cin + ci0 + ci) * NN + t]);
            wl[e] = v;
        }
        __syncthreads();
        if (!valid) continue;
        const int nci = a.Cin - ci0 < CI_CH ? a.Cin - ci0 : CI_CH;
        for (int ci = 0; ci < nci; ++ci) {
            const TIn* xp = x + ((size_t)b * a.Cin + ci0 + ci) * a.H * a.W;
            for (int u = 0; u < Tr; ++u) {
                const int i = i0 + u * xstep;
                if (i < 0 || i >= a.H) continue;
                for (int v = 0; v < Tc; ++v) {
                    const int j = j0 + v * xstep;
                    if (j < 0 || j >= a.W) continue;
                    const float xv = to_f32(xp[(size_t)i * a.W + j]);
                    const int tap = (r + u * wstep) * n + (c + v * wstep);
                    const float4* wp = reinterpret_cast<const float4*>(&wl[(ci * NN + tap) * CO_BLK]);
                    const float4 w0 = wp[0], w1 = wp[1];
                    acc[0] = fmaf(xv, w0.x, acc[0]); acc[1] = fmaf(xv, w0.y, acc[1]);
                    acc[2] = fmaf(xv, w0.z, acc[2]); acc[3] = fmaf(xv, w0.w, acc[3]);
                    acc[4] = fmaf(xv, w1.x, acc[4]); acc[5] = fmaf(xv, w1.y, acc[5]);
                    acc[6] = fmaf(xv, w1.z, acc[6]); acc[7] = fmaf(xv, w1.w, acc[7]);
                }
            }
        }
    }
    if (!valid) return;
#pragma unroll
    for (int co = 0; co < CO_BLK; ++co)
        if (co0 + co < a.Cout)
            y[(((size_t)b * a.Cout + co0 + co) * a.OH + oy) * a.OW + ox] = acc[co];
}

}  // namespace

// k = stride (dilated == 0) or dilation (dilated == 1); shapes validated by the caller
hipError_t launch_general(int dilated, int B, int Cin, int Cout, int H, int W, int n, int P, int k,
                          int OH, int OW, const void* x, const void* w, float* y, int dtype,
                          hipStream_t stream)
{
    GenArgs a;
    a.B = B; a.Cin = Cin; a.Cout = Cout; a.H = H; a.W = W; a.n = n; a.P = P; a.k = k;
    a.OH = OH; a.OW = OW; a.dilated = dilated;
    a.tilesX = (OW + 31) / 32;
    a.tilesY = (OH + 7) / 8;
    a.coBlocks = (Cout + CO_BLK - 1) / CO_BLK;
    const long long nb = (long long)a.tilesX * a.tilesY * a.coBlocks * B;
    if (nb > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    if (dtype == 0)
        hipLaunchKernelGGL(ukst_general_kernel<float>, dim3((unsigned)nb), dim3(256), 0, stream,
                           (const float*)x, (const float*)w, y, a);
    else
        hipLaunchKernelGGL(ukst_general_kernel<uint16_t>, dim3((unsigned)nb), dim3(256), 0, stream,
                           (const uint16_t*)x, (const uint16_t*)w, y, a);
    return hipGetLastError();
}

}  // namespace ukst
