// Thin-output path (fp32, Cout <= 4, any Cin > 4): the last layer of a generator, e.g. 64 -> 3
// channels.  The work is a long reduction over input channels into very few outputs, so it runs on
// the vector ALUs like the narrow-channel kernel, with the same lane layout: a lane owns 4
// consecutive output columns (a 16-byte aligned group counted from column 0) by 2*QH output rows,
// for every output channel, and the four parity classes of Algorithm 2 appear as compile-time
// constants (output column c uses the taps of column parity (c + P) & 1, output row class r the
// taps of row parity r, Sec. 3.1-3.2): every tap is used exactly once per output it belongs to.
//
// Small maps do not fill 64 lanes along a row, so the lanes of a wave are folded into LW column
// groups by 64/LW row bands.  The four waves of a block work on the SAME outputs and split the
// input channels between them (each walks Cin/4 channels, the window of the next channel being
// requested while the current one is multiplied); the partial sums meet in LDS and wave 0 writes
// them, one 16-byte store per row and lane.
//
// Edges are handled by the buffer addressing hardware: a window element that does not exist (row
// or column outside the map: the floor(P/2) zero padding of Sec. 3.4) gets a byte offset beyond
// the descriptor of its channel plane and loads as 0; an output row that does not exist gets
// such an offset for its store, which is dropped.  Rows differ between the lanes of a wave here,
// so the size field cannot clip a row end as it does in the narrow kernel: a column group that
// sticks out of an output row is written column by column.
#include "ukst_internal.h"

namespace ukst {
namespace {

typedef unsigned u2v __attribute__((ext_vector_type(2)));
typedef unsigned u3v __attribute__((ext_vector_type(3)));
typedef unsigned u4v __attribute__((ext_vector_type(4)));

constexpr int kRsrcFlags = 0x00020000;       // raw 32-bit buffer, gfx9 family
constexpr unsigned kNoColumn = 0x80000000u;  // beyond the size field of any row (images < 1 GiB)
constexpr int kFarBand = 0x20000000;         // a quad row whose input and output rows do not exist
constexpr int kMaxWeightFloats = 8192;       // 32 KiB of LDS for the block's weights

__device__ __forceinline__ unsigned fbits(float f) { return __builtin_bit_cast(unsigned, f); }

template <int N, int CO, int QH, bool PE>
__global__ __launch_bounds__(256) void ukst_thin_kernel(const float* __restrict__ x,
                                                       const float* __restrict__ w,
                                                       float* __restrict__ y, GeomBase g, int lwlog,
                                                       int strips, int bgroups, int nblocks,
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
    constexpr int NACC = CO * QH * 2 * 4;  // partial sums per lane
    extern __shared__ __align__(16) float smem[];  // weights [Cin][CO][NNP], then the reduction
    float* wl = smem;
    float* red = smem + g.Cin * CO * NNP;  // [3 waves][NACC][64 lanes]

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // which quarter of the input channels
    const int lane = tid & 63;
    int bid = blockIdx.x;
    const int strip = bid % strips; bid /= strips;
    const int bgroup = bid % bgroups;
    const int b = bid / bgroups;

    const int H = g.H, W = g.W, P = g.P, OH = g.OH, OW = g.OW, Cin = g.Cin;
    const int lx = lane & ((1 << lwlog) - 1), ly = lane >> lwlog;
    const int lg = (strip << lwlog) + lx;                       // the lane's column group
    const int band = bgroup * (64 >> lwlog) + ly;                // the lane's band of QH quad rows
    const int k0 = (band * QH < g.KH) ? g.k_min + band * QH : kFarBand;
    const int j0 = 2 * lg - (P >> 1);                            // first input column of the window
    const int i0 = k0 - P;                                       // first input row of the window

    // One load fetches the lane's WC consecutive window columns of a row (the address unit takes
    // as long for 4 bytes as for 16).  The descriptor ends with the channel plane, so columns
    // outside the map are not clipped by the hardware here: a lane whose window starts left of
    // the map loads from column 0 and shifts, and elements right of the map are zeroed, both
    // with per-lane masks computed once.  A missing row gets an offset beyond any plane.
    const int left = j0 < 0 ? (-j0 < WC ? -j0 : WC) : 0;  // window columns left of the map
    const unsigned woff = j0 < 0 ? 0u : (unsigned)j0 * 4u;
    bool keep[WC];                                         // column exists (after the shift)
#pragma unroll
    for (int v = 0; v < WC; ++v) keep[v] = j0 + v >= 0 && j0 + v < W;
    unsigned roff[WR];
#pragma unroll
    for (int u = 0; u < WR; ++u) {
        const int i = i0 + u;
        roff[u] = (i >= 0 && i < H && j0 < W) ? (unsigned)i * (unsigned)W * 4u + woff : kNoColumn;
    }

    const float* xb = x + (size_t)b * Cin * H * W;
    const unsigned xrow = (unsigned)W * 4u, xplane = (unsigned)H * xrow;
    const int cps = (Cin + 3) >> 2;                 // channels per wave
    const int ci_begin = wave * cps;
    const int ci_end = (ci_begin + cps < Cin) ? ci_begin + cps : Cin;
    const bool any_left = __builtin_amdgcn_ballot_w64(left > 0) != 0;  // wave-uniform
    auto load_window = [&](int ci, unsigned (&raw)[WR][WC]) {
        const bool ok = ci < ci_end;  // wave-uniform
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            (void*)xb, 0, ok ? (int)((unsigned)(ci + 1) * xplane) : 0, kRsrcFlags);
        const unsigned start = (unsigned)ci * xplane;
#pragma unroll
        for (int u = 0; u < WR; ++u) {
            // elements by value: a bit cast of a vector element reads element 0
            if constexpr (WC == 4) {
                const u4v t = __builtin_amdgcn_raw_buffer_load_b128(rs, roff[u], start, 0);
                raw[u][0] = t.x; raw[u][1] = t.y; raw[u][2] = t.z; raw[u][3] = t.w;
            } else if constexpr (WC == 3) {
                const u3v t = __builtin_amdgcn_raw_buffer_load_b96(rs, roff[u], start, 0);
                raw[u][0] = t.x; raw[u][1] = t.y; raw[u][2] = t.z;
            } else {
                const u2v t = __builtin_amdgcn_raw_buffer_load_b64(rs, roff[u], start, 0);
                raw[u][0] = t.x; raw[u][1] = t.y;
            }
        }
    };
    // raw window -> window: shift right by `left` columns, zero what lies outside the map
    auto fix_window = [&](const unsigned (&raw)[WR][WC], float (&win)[WR][WC]) {
#pragma unroll
        for (int u = 0; u < WR; ++u) {
            unsigned e[WC];
#pragma unroll
            for (int v = 0; v < WC; ++v) e[v] = raw[u][v];
            if (any_left) {
#pragma unroll
                for (int s = 1; s <= WC; ++s) {
                    const bool m = left >= s;
#pragma unroll
                    for (int v = WC - 1; v >= 1; --v) e[v] = m ? e[v - 1] : e[v];
                }
            }
#pragma unroll
            for (int v = 0; v < WC; ++v) win[u][v] = keep[v] ? __uint_as_float(e[v]) : 0.f;
        }
    };

    float acc[CO][QH][2][4];
#pragma unroll
    for (int co = 0; co < CO; ++co)
#pragma unroll
        for (int qy = 0; qy < QH; ++qy)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[co][qy][0][c] = acc[co][qy][1][c] = 0.f;

    auto accumulate = [&](int ci, const float (&win)[WR][WC]) {
#pragma unroll
        for (int co = 0; co < CO; ++co) {
            float wv[NNP];
#pragma unroll
            for (int t = 0; t < NNP; t += 4) {
                const float4 q = *reinterpret_cast<const float4*>(&wl[(ci * CO + co) * NNP + t]);
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
                                acc[co][qy][a & 1][c] = fmaf(win[qy + (a >> 1)][jr + (t >> 1)],
                                                             wv[a * N + t], acc[co][qy][a & 1][c]);
                        }
        }
    };

    // first window in flight, then the block's weights: [ci][co][tap] in LDS, padded taps zero
    unsigned rawA[WR][WC], rawB[WR][WC];
    float win[WR][WC];
    load_window(ci_begin, rawA);
    __builtin_amdgcn_sched_barrier(0);
    for (int e = tid; e < Cin * CO * NNP; e += 256) {
        const int t = e % NNP, pair = e / NNP;  // pair = ci * CO + co
        const int co = pair % CO, ci = pair / CO;
        wl[e] = (t < NN) ? w[((size_t)co * Cin + ci) * NN + t] : 0.f;
    }
    __syncthreads();

    // channels two at a time so that the two window buffers keep their names; a channel past the
    // wave's share loads zeros and is not multiplied
    for (int ci = ci_begin; ci < ci_end; ci += 2) {
        load_window(ci + 1, rawB);
        fix_window(rawA, win);
        accumulate(ci, win);
        load_window(ci + 2, rawA);
        if (ci + 1 < ci_end) {
            fix_window(rawB, win);
            accumulate(ci + 1, win);
        }
    }

    // ---- the four partial sums of every output meet in LDS; wave 0 adds and stores
    if (wave > 0) {
        float* dst = red + (size_t)(wave - 1) * NACC * 64 + lane;
        int e = 0;
#pragma unroll
        for (int co = 0; co < CO; ++co)
#pragma unroll
            for (int qy = 0; qy < QH; ++qy)
#pragma unroll
                for (int r = 0; r < 2; ++r)
#pragma unroll
                    for (int c = 0; c < 4; ++c) dst[(e++) * 64] = acc[co][qy][r][c];
    }
    __syncthreads();
    if (wave > 0) return;
    {
        int e = 0;
#pragma unroll
        for (int co = 0; co < CO; ++co)
#pragma unroll
            for (int qy = 0; qy < QH; ++qy)
#pragma unroll
                for (int r = 0; r < 2; ++r)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        acc[co][qy][r][c] += red[(0 * NACC + e) * 64 + lane] +
                                             red[(1 * NACC + e) * 64 + lane] +
                                             red[(2 * NACC + e) * 64 + lane];
                        ++e;
                    }
    }

    if (has_epilogue(ep)) {  // uniform
#pragma unroll
        for (int co = 0; co < CO; ++co) {
            const float bv = ep.bias ? ep.bias[co] : 0.f;
#pragma unroll
            for (int qy = 0; qy < QH; ++qy)
#pragma unroll
                for (int r = 0; r < 2; ++r)
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        acc[co][qy][r][c] = epilogue(acc[co][qy][r][c], bv, ep.act);
        }
    }

    float* yb = y + (size_t)b * CO * OH * OW;
    const unsigned yrow = (unsigned)OW * 4u, yplane = (unsigned)OH * yrow;
    const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(
        (void*)yb, 0, (int)((unsigned)CO * yplane), kRsrcFlags);
    // rows differ between lanes, so the row end cannot clip a store through the size field: a
    // lane whose four columns are not all inside the row stores them one by one
    const int ox0 = 4 * lg;
    const bool whole = ox0 + 3 < OW;
#pragma unroll
    for (int co = 0; co < CO; ++co)
#pragma unroll
        for (int qy = 0; qy < QH; ++qy)
#pragma unroll
            for (int r = 1; r >= 0; --r) {
                const int oy = 2 * (k0 + qy) - P - r;  // row class r of quad row k0 + qy
                const bool rowok = oy >= 0 && oy < OH;
                const unsigned at = (unsigned)co * yplane + (unsigned)oy * yrow + (unsigned)ox0 * 4u;
                u4v d;
                d.x = fbits(acc[co][qy][r][0]); d.y = fbits(acc[co][qy][r][1]);
                d.z = fbits(acc[co][qy][r][2]); d.w = fbits(acc[co][qy][r][3]);
                __builtin_amdgcn_raw_buffer_store_b128(d, rs_y, (rowok && whole) ? at : kNoColumn, 0, 0);
                if (__builtin_amdgcn_ballot_w64(rowok && !whole && ox0 < OW) != 0) {  // wave-uniform
                    const bool part = rowok && !whole;
                    __builtin_amdgcn_raw_buffer_store_b32(d.x, rs_y, (part && ox0 < OW) ? at : kNoColumn, 0, 0);
                    __builtin_amdgcn_raw_buffer_store_b32(d.y, rs_y, (part && ox0 + 1 < OW) ? at + 4u : kNoColumn, 0, 0);
                    __builtin_amdgcn_raw_buffer_store_b32(d.z, rs_y, (part && ox0 + 2 < OW) ? at + 8u : kNoColumn, 0, 0);
                }
            }
}

template <int N, int CO, int QH, bool PE>
hipError_t launch_q(const Geom& g, const float* x, const float* w, float* y, hipStream_t stream)
{
    constexpr int NNP = (N * N + 3) & ~3;
    const int groups = (g.OW + 3) / 4;                    // column groups per row
    const int lwlog = groups <= 8 ? 3 : groups <= 16 ? 4 : groups <= 32 ? 5 : 6;
    const int strips = (groups + (1 << lwlog) - 1) >> lwlog;
    const int bands = (g.KH + QH - 1) / QH;
    const int per_wave = 64 >> lwlog;                     // bands folded into one wave
    const int bgroups = (bands + per_wave - 1) / per_wave;
    const long long nblocks = (long long)strips * bgroups * g.B;
    if (nblocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const size_t lds = ((size_t)g.Cin * CO * NNP + 3 * (size_t)(CO * QH * 8) * 64) * sizeof(float);
    hipLaunchKernelGGL((ukst_thin_kernel<N, CO, QH, PE>), dim3((unsigned)nblocks), dim3(256), lds,
                       stream, x, w, y, (GeomBase)g, lwlog, strips, bgroups, (int)nblocks, g.ep);
    return hipGetLastError();
}

template <int N, int CO>
hipError_t launch_p(const Geom& g, const float* x, const float* w, float* y, hipStream_t stream)
{
    return (g.P & 1) ? launch_q<N, CO, 1, false>(g, x, w, y, stream)
                     : launch_q<N, CO, 1, true>(g, x, w, y, stream);
}

template <int N>
hipError_t launch_co(const Geom& g, const float* x, const float* w, float* y, hipStream_t st)
{
    switch (g.Cout) {
        case 1: return launch_p<N, 1>(g, x, w, y, st);
        case 2: return launch_p<N, 2>(g, x, w, y, st);
        case 3: return launch_p<N, 3>(g, x, w, y, st);
        case 4: return launch_p<N, 4>(g, x, w, y, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool thin_supported(const Geom& g, int dtype)
{
    // 32-bit byte offsets inside the image of one batch item, with room for the out-of-range
    // marker; weights of the whole layer in LDS next to the reduction buffer (under 64 KiB together)
    const long long xbytes = 4LL * g.Cin * g.H * g.W, ybytes = 4LL * g.Cout * g.OH * g.OW;
    const int nnp = (g.n * g.n + 3) & ~3;
    return dtype == 0 && g.Cout <= 4 && g.Cin > 4 && g.n >= 2 && g.n <= 5 && xbytes < (1LL << 30) &&
           ybytes < (1LL << 30) && g.P < (1 << 20) &&
           (long long)g.Cin * g.Cout * nnp <= kMaxWeightFloats;
}

hipError_t launch_thin(const Geom& g, const void* x, const void* w, float* y, hipStream_t stream)
{
    const float* xf = (const float*)x;
    const float* wf = (const float*)w;
    switch (g.n) {
        case 2: return launch_co<2>(g, xf, wf, y, stream);
        case 3: return launch_co<3>(g, xf, wf, y, stream);
        case 4: return launch_co<4>(g, xf, wf, y, stream);
        case 5: return launch_co<5>(g, xf, wf, y, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ukst
