// Backward pass of the stride-2 transpose convolution: the two gradients of the linear map of
// Algorithm 1 / Algorithm 2, evaluated like the forward pass without ever touching an inserted
// zero.  (The paper measures the forward layer only; training a generator needs these too.)
//
// The same parity argument as in Sec. 3.1 applies in reverse: input pixel (i, j) meets output
// pixel (oy, ox) through tap (a, c) = (2i + P - oy, 2j + P - ox), so tap row a only ever pairs an
// input row with output rows of parity (P - a) & 1.  Hence
//
//   dx[b,ci,i,j]  = sum_co sum_{a,c<n} dy[b,co,2i+P-a,2j+P-c] * w[co,ci,a,c]
//   dw[co,ci,a,c] = sum_b  sum_{i,j}   x[b,ci,i,j] * dy[b,co,2i+P-a,2j+P-c]
//
// (terms whose output pixel lies outside [0,OH) x [0,OW) drop out): every input pixel gathers from
// a stride-2 lattice of dy, each of the n*n taps is used once per pixel, and the number of
// multiply-adds equals that of the forward pass.  Both kernels stage dy tiles in LDS with rows
// that fall outside the output filled with zeros, which is the predicate of the formulas above.
#include "ukst_internal.h"

namespace ukst {
namespace {

__device__ __forceinline__ float ld_f32(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float ld_f32(const uint16_t* p, size_t i) { return __uint_as_float((uint32_t)p[i] << 16); }

// Staging loop of a 256-thread block: element e = tid, tid + 256, ... < total is fetched with
// fetch(e, dst) -> value (dst = its LDS index) and written to lds[dst].  The loads of U
// elements are all issued before the first is stored, so their latencies overlap instead of
// adding up.
template <int U, class Fetch>
__device__ __forceinline__ void stage_elements(float* lds, int tid, int total, Fetch fetch)
{
    for (int e0 = tid; e0 < total; e0 += 256 * U) {
        float v[U];
        int dst[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + 256 * u;
            dst[u] = -1;
            v[u] = 0.f;
            if (e < total) v[u] = fetch(e, dst[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (dst[u] >= 0) lds[dst[u]] = v[u];
    }
}

// Four consecutive elements starting at element index i (any element alignment).
struct Quad { float v[4]; };
__device__ __forceinline__ Quad ld_quad(const float* p, size_t i)
{
    typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
    const f4u t = *reinterpret_cast<const f4u*>(p + i);
    return Quad{{t[0], t[1], t[2], t[3]}};
}
__device__ __forceinline__ Quad ld_quad(const uint16_t* p, size_t i)
{
    typedef unsigned u2u __attribute__((ext_vector_type(2), aligned(2)));
    const u2u t = *reinterpret_cast<const u2u*>(p + i);
    return Quad{{__uint_as_float(t[0] << 16), __uint_as_float(t[0] & 0xFFFF0000u),
                 __uint_as_float(t[1] << 16), __uint_as_float(t[1] & 0xFFFF0000u)}};
}

// Stages the parity-split dy tile of a block: `nrows` rows (row = (channel, image, dy row), the
// last two as rowsPerCo = TB * LR per channel), `cols` columns each.  A thread moves four
// consecutive columns with one vector load (scalar loads where the four straddle the edge of the
// tensor), columns or rows outside the output become zeros; the loads of U quads are issued
// before the first is stored.  LDS position of column cc of a row: (cc & 1) * HC + (cc >> 1).
struct DyTile {
    int nrows, rowsPerCo, coStride, cols, cols4, HC, LR;
    int co_first, co_end, b0, oy_base, ox_base;
    FastDiv dC4, dRowsPerCo, dLR;
};
template <int U, typename TIn>
__device__ __forceinline__ void stage_dy_tile(float* lds, const TIn* __restrict__ dy, const GeomBase& g,
                                              const DyTile& t, int tid)
{
    const int n = t.nrows * t.cols4;
    for (int e0 = tid; e0 < n; e0 += 256 * U) {
        Quad q[U];
        int dst[U], ncol[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + 256 * u;
            dst[u] = -1;
            q[u] = Quad{{0.f, 0.f, 0.f, 0.f}};
            if (e < n) {
                const int row = fdiv(e, t.dC4), cc = 4 * (e - row * t.cols4);
                const int col = fdiv(row, t.dRowsPerCo), rem = row - col * t.rowsPerCo;
                const int bl = fdiv(rem, t.dLR), rr = rem - bl * t.LR;
                const int b = t.b0 + bl, co = t.co_first + col, oy = t.oy_base + rr, ox = t.ox_base + cc;
                dst[u] = col * t.coStride + rem * t.cols + (cc >> 1);
                ncol[u] = t.cols - cc;  // columns of this quad that belong to the row (2 or >= 4)
                if (co < t.co_end && b < g.B && oy >= 0 && oy < g.OH && ox + 3 >= 0 && ox < g.OW) {
                    const size_t src = (((size_t)b * g.Cout + co) * g.OH + oy) * g.OW;
                    if (ox >= 0 && ox + 3 < g.OW) {
                        q[u] = ld_quad(dy, src + ox);
                    } else {
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (ox + k >= 0 && ox + k < g.OW) q[u].v[k] = ld_f32(dy, src + ox + k);
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (dst[u] >= 0) {
                lds[dst[u]] = q[u].v[0];
                lds[dst[u] + t.HC] = q[u].v[1];
                if (ncol[u] > 2) {
                    lds[dst[u] + 1] = q[u].v[2];
                    lds[dst[u] + t.HC + 1] = q[u].v[3];
                }
            }
    }
}

// ------------------------------------------------------------------------------------------
// Gradient with respect to the input.
//
// Block = 256 threads = TJ pixel columns x 256/TJ thread rows; a thread owns PX pixels (thread
// rows 256/TJ apart) x CI_BLK input channels.  Thread rows enumerate (image, pixel row) pairs of
// a tile of TB images x TI rows, so that small maps still fill the block.  Per chunk of output
// channels the dy rows under the tile go to LDS, split by column parity so that the stride-2
// lattice a wave reads is contiguous: dy column 2*j0 + P - (n-1) + cc sits at [cc & 1][cc >> 1].
// The weights of the chunk go to LDS as [co][tap][CI_BLK] and are read as 16-byte broadcasts.
struct GradInArgs {
    GeomBase g;
    int TJ, TI, TB;            // tile: pixel columns, pixel rows, images (powers of two)
    int logTJ, logTI;
    int LR, HC;                // staged dy rows per image, staged columns per parity
    int tilesX, tilesY, tilesB, ciBlocks;
    int coChunk;               // output channels staged per round
    int cols4;                 // four-column pieces per staged dy row
    FastDiv dC4, dRowsPerCo, dLR;
};

template <int N, int CI_BLK, int PX, typename TIn>
__global__ __launch_bounds__(256) void ukst_grad_input_kernel(const TIn* __restrict__ dy,
                                                             const TIn* __restrict__ w,
                                                             float* __restrict__ dx, GradInArgs a)
{
    constexpr int NN = N * N;
    extern __shared__ __align__(16) float lds_f[];
    const GeomBase& g = a.g;
    const int tid = threadIdx.x;
    const int tileFloats = a.TB * a.LR * 2 * a.HC;  // per output channel
    float* wl = lds_f;                               // [coChunk][NN][CI_BLK]
    float* tile = lds_f + a.coChunk * NN * CI_BLK;   // [coChunk][TB][LR][2][HC]

    int bid = xcd_contiguous(blockIdx.x, gridDim.x);     // neighbours in this numbering share an L2
    const int cb = bid % a.ciBlocks; bid /= a.ciBlocks;  // blocks that share a dy tile are neighbours
    const int tx = bid % a.tilesX; bid /= a.tilesX;
    const int ty = bid % a.tilesY; bid /= a.tilesY;
    const int tb = bid;
    const int ci0 = cb * CI_BLK, i0 = ty * a.TI, j0 = tx * a.TJ, b0 = tb * a.TB;
    const int oy_base = 2 * i0 + g.P - (N - 1), ox_base = 2 * j0 + g.P - (N - 1);

    const int lj = tid & (a.TJ - 1), trow = tid >> a.logTJ, rowStep = 256 >> a.logTJ;
    int toff[PX];  // LDS offset of the pixel's (image, 2*row) origin inside a channel's tile
#pragma unroll
    for (int p = 0; p < PX; ++p) {
        const int tr = trow + p * rowStep;
        const int bl = tr >> a.logTI, li = tr & (a.TI - 1);
        toff[p] = ((bl * a.LR + 2 * li) * 2) * a.HC + lj;
    }
    float acc[PX][CI_BLK];
#pragma unroll
    for (int p = 0; p < PX; ++p)
#pragma unroll
        for (int q = 0; q < CI_BLK; ++q) acc[p][q] = 0.f;

    const int rowsPerCo = a.TB * a.LR, cols = 2 * a.HC;
    for (int co0 = 0; co0 < g.Cout; co0 += a.coChunk) {
        const int nco = g.Cout - co0 < a.coChunk ? g.Cout - co0 : a.coChunk;
        if (co0) __syncthreads();
        // weights of the chunk: wl[co][tap][q] = w[co0+co][ci0+q][tap], zero beyond Cin
        stage_elements<4>(wl, tid, nco * NN * CI_BLK, [&](int e, int& dst) {
            const int q = e % CI_BLK, t = (e / CI_BLK) % NN, co = e / (CI_BLK * NN);
            dst = e;
            return (ci0 + q < g.Cin)
                       ? ld_f32(w, ((size_t)(co0 + co) * g.Cin + ci0 + q) * NN + t) : 0.f;
        });
        // dy rows under the tile, lanes along the columns; rows or columns outside the output (and
        // images beyond the batch) are zeros
        {
            DyTile t;
            t.nrows = nco * rowsPerCo; t.rowsPerCo = rowsPerCo; t.coStride = tileFloats; t.cols = cols;
            t.cols4 = a.cols4; t.HC = a.HC; t.LR = a.LR; t.co_first = co0; t.co_end = g.Cout; t.b0 = b0;
            t.oy_base = oy_base; t.ox_base = ox_base; t.dC4 = a.dC4; t.dRowsPerCo = a.dRowsPerCo; t.dLR = a.dLR;
            stage_dy_tile<4>(tile, dy, g, t, tid);
        }
        __syncthreads();
        for (int co = 0; co < nco; ++co) {
            const float* tc = tile + co * tileFloats;
            const float* wc = wl + co * NN * CI_BLK;
#pragma unroll
            for (int ta = 0; ta < N; ++ta)
#pragma unroll
                for (int tcx = 0; tcx < N; ++tcx) {
                    // tap (ta, tcx): dy row 2*li + (N-1-ta), dy column 2*lj + (N-1-tcx)
                    const int off = ((N - 1 - ta) * 2 + ((N - 1 - tcx) & 1)) * a.HC + ((N - 1 - tcx) >> 1);
                    float wv[CI_BLK];
#pragma unroll
                    for (int q4 = 0; q4 < CI_BLK; q4 += 4) {
                        const float4 t4 = *reinterpret_cast<const float4*>(wc + (ta * N + tcx) * CI_BLK + q4);
                        wv[q4] = t4.x; wv[q4 + 1] = t4.y; wv[q4 + 2] = t4.z; wv[q4 + 3] = t4.w;
                    }
#pragma unroll
                    for (int p = 0; p < PX; ++p) {
                        const float d = tc[toff[p] + off];
#pragma unroll
                        for (int q = 0; q < CI_BLK; ++q) acc[p][q] = fmaf(d, wv[q], acc[p][q]);
                    }
                }
        }
    }

    const int j = j0 + lj;
#pragma unroll
    for (int p = 0; p < PX; ++p) {
        const int tr = trow + p * rowStep;
        const int b = b0 + (tr >> a.logTI), i = i0 + (tr & (a.TI - 1));
        if (b >= g.B || i >= g.H || j >= g.W) continue;
#pragma unroll
        for (int q = 0; q < CI_BLK; ++q)
            if (ci0 + q < g.Cin) dx[(((size_t)b * g.Cin + ci0 + q) * g.H + i) * g.W + j] = acc[p][q];
    }
}

int log2_of(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }
int pow2_ceil(int v) { return 1 << log2_of(v); }

template <int N, int CI_BLK, int PX, typename TIn>
hipError_t launch_gi(const Geom& g, const void* dy, const void* w, float* dx, hipStream_t stream)
{
    GradInArgs a;
    a.g = g;
    a.TJ = pow2_ceil(g.W < 32 ? g.W : 32);
    if (a.TJ < 4) a.TJ = 4;
    const int TR = PX * 256 / a.TJ;
    a.TI = pow2_ceil(g.H < TR ? g.H : TR);
    a.TB = TR / a.TI;
    a.logTJ = log2_of(a.TJ);
    a.logTI = log2_of(a.TI);
    a.LR = 2 * a.TI + N - 2 > 1 ? 2 * a.TI + N - 2 : 1;
    a.HC = a.TJ + N / 2;
    a.tilesX = (g.W + a.TJ - 1) / a.TJ;
    a.tilesY = (g.H + a.TI - 1) / a.TI;
    a.tilesB = (g.B + a.TB - 1) / a.TB;
    a.ciBlocks = (g.Cin + CI_BLK - 1) / CI_BLK;
    const size_t tileBytes = (size_t)a.TB * a.LR * 2 * a.HC * 4, wBytes = (size_t)N * N * CI_BLK * 4;
    const size_t budget = 64 * 1024;
    int cc = (int)(budget / (tileBytes + wBytes));
    if (cc < 1) return hipErrorInvalidConfiguration;  // cannot happen for n <= 7 (a channel's tile stays below 51 KiB)
    if (cc > 8) cc = 8;
    if (cc > g.Cout) cc = g.Cout;
    a.coChunk = cc;
    a.cols4 = (2 * a.HC + 3) / 4;
    a.dC4 = make_fastdiv((unsigned)a.cols4);
    a.dRowsPerCo = make_fastdiv((unsigned)(a.TB * a.LR));
    a.dLR = make_fastdiv((unsigned)a.LR);
    const long long nb = (long long)a.tilesX * a.tilesY * a.tilesB * a.ciBlocks;
    if (nb > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const size_t lds = (size_t)cc * (tileBytes + wBytes);
    hipLaunchKernelGGL((ukst_grad_input_kernel<N, CI_BLK, PX, TIn>), dim3((unsigned)nb), dim3(256), lds,
                       stream, (const TIn*)dy, (const TIn*)w, dx, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Gradient with respect to the input on the matrix cores (wide layers, either dtype).
//
// The gather above is one dense product per tap: D[ci][pixel] += sum_co W_tap[ci][co] *
// DY_tap[co][pixel], DY_tap being dy on the tap's stride-2 lattice.  v_mfma_f32_32x32x2_f32 takes
// 32 input channels x 32 pixels of one tile row x two output channels per instruction; an fp32
// MFMA lane holds a single K value per operand, so both fragments are plain 4-byte LDS reads of
// consecutive addresses: the weights from a copy packed once per call as [co][tap][ci] (fp32,
// zero padded), dy from the same parity-split tile as the vector-ALU kernel.  bf16 operands are
// widened to fp32 on their way into LDS (exact), so one kernel serves both element types.
// Block = 4 waves = WM (channel halves) x WP (row groups); wave tile 64 channels x 4 tile rows of
// 32 pixels = 8 accumulator tiles; two blocks per compute unit cover each other's staging.
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct GiMfmaArgs {
    GeomBase g;
    int WM, logWM;             // waves along the input channels (1 or 2)
    int CI_T, logC4, WS;       // channels per block, log2(CI_T / 4), LDS row stride of a tap's channels
    int CIp, CoutP;            // padded sizes of the packed weights
    int TJ, logTJ;             // pixel columns per tile (4..32): the 32 MFMA columns hold 32/TJ tile rows
    int TI, TB, logTI;         // tile rows are (image, pixel row) pairs: TB images x TI rows
    int LR, HC;
    int tilesX, tilesY, tilesB, ciTiles;
    int CC;                    // output channels per LDS round (even)
    int KS, coPer;             // slices of the output-channel sum (grid.y) and channels per slice
    int cols4;                 // four-column pieces per staged dy row
    FastDiv dC4, dRowsPerCo, dLR;
};

template <typename TIn>
__global__ __launch_bounds__(256) void ukst_pack_w_kernel(const TIn* __restrict__ w, float* __restrict__ wp,
                                                         int Cout, int Cin, int NN, int CoutP, int CIp)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)CoutP * NN * CIp) return;
    const int ci = (int)(idx % CIp);
    const size_t row = idx / CIp;
    const int tap = (int)(row % NN), co = (int)(row / NN);
    float v = 0.f;
    if (co < Cout && ci < Cin) v = ld_f32(w, ((size_t)co * Cin + ci) * NN + tap);
    wp[idx] = v;
}

template <int N, typename TIn>
__global__ __launch_bounds__(256, 2) void ukst_grad_input_mfma_kernel(const TIn* __restrict__ dy,
                                                                     const float* __restrict__ wp,
                                                                     float* __restrict__ dx, GiMfmaArgs a)
{
    constexpr int NN = N * N;
    extern __shared__ __align__(16) float lds_f[];
    const GeomBase& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kk = lane >> 5;
    const int wm = wave & (a.WM - 1), wpx = wave >> a.logWM;
    const int wlStride = NN * a.WS;                      // floats per output channel
    const int tileFloats = a.TB * a.LR * 2 * a.HC;
    float* wl = lds_f;                                   // [CC][NN][WS]
    float* tile = lds_f + a.CC * wlStride;               // [CC][TB][LR][2][HC]

    // neighbours in this numbering share an L2; the slices of a split sum (grid.y) come last
    const int lin = xcd_contiguous(blockIdx.y * gridDim.x + blockIdx.x, gridDim.x * gridDim.y);
    const int ks = lin / gridDim.x;
    int bid = lin - ks * gridDim.x;
    const int cit = bid % a.ciTiles; bid /= a.ciTiles;   // blocks that share a dy tile are neighbours
    const int tx = bid % a.tilesX; bid /= a.tilesX;
    const int ty = bid % a.tilesY; bid /= a.tilesY;
    const int tb = bid;
    const int ci0 = cit * a.CI_T, i0 = ty * a.TI, j0 = tx * a.TJ, b0 = tb * a.TB;
    const int oy_base = 2 * i0 + g.P - (N - 1), ox_base = 2 * j0 + g.P - (N - 1);

    // MFMA column l32 = (tile row within the group, pixel column): narrow maps put several rows
    // side by side so that all 32 columns carry pixels
    const int lj = l32 & (a.TJ - 1), lsub = l32 >> a.logTJ, subRows = 32 >> a.logTJ;
    int toff[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int tr = (wpx * 4 + t) * subRows + lsub;
        const int bl = tr >> a.logTI, li = tr & (a.TI - 1);
        toff[t] = kk * tileFloats + ((bl * a.LR + 2 * li) * 2) * a.HC + lj;
    }
    const int a_base = kk * wlStride + wm * 64 + l32;
    f32x16 acc[2][4];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][t][i] = 0.f;

    const int rowsPerCo = a.TB * a.LR, cols = 2 * a.HC;
    const int c4n = 1 << a.logC4;  // float4 pieces per weight row
    const int co_begin = ks * a.coPer;
    const int co_end = co_begin + a.coPer < a.CoutP ? co_begin + a.coPer : a.CoutP;
    for (int co0 = co_begin; co0 < co_end; co0 += a.CC) {
        if (co0 != co_begin) __syncthreads();
        // packed weights of the round: eight 16-byte pieces in flight per thread; no predicates
        // (a written-out loop waits for every load): indices past the end repeat the last piece
        {
            const int npc = a.CC * NN * c4n;
            for (int e0 = tid; e0 < npc; e0 += 256 * 8) {
                float4 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = e0 + 256 * u < npc ? e0 + 256 * u : npc - 1;
                    v[u] = *reinterpret_cast<const float4*>(
                        wp + ((size_t)co0 * NN + (e >> a.logC4)) * a.CIp + ci0 + 4 * (e & (c4n - 1)));
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = e0 + 256 * u < npc ? e0 + 256 * u : npc - 1;
                    *reinterpret_cast<float4*>(wl + (e >> a.logC4) * a.WS + 4 * (e & (c4n - 1))) = v[u];
                }
            }
        }
        {
            DyTile t;
            t.nrows = a.CC * rowsPerCo; t.rowsPerCo = rowsPerCo; t.coStride = tileFloats; t.cols = cols;
            t.cols4 = a.cols4; t.HC = a.HC; t.LR = a.LR; t.co_first = co0; t.co_end = g.Cout; t.b0 = b0;
            t.oy_base = oy_base; t.ox_base = ox_base; t.dC4 = a.dC4; t.dRowsPerCo = a.dRowsPerCo; t.dLR = a.dLR;
            stage_dy_tile<4>(tile, dy, g, t, tid);
        }
        __syncthreads();
        for (int cp = 0; cp < a.CC; cp += 2) {
            const float* wa = wl + cp * wlStride + a_base;
            const float* tc = tile + cp * tileFloats;
#pragma unroll
            for (int ta = 0; ta < N; ++ta)
#pragma unroll
                for (int tcx = 0; tcx < N; ++tcx) {
                    const int off = ((N - 1 - ta) * 2 + ((N - 1 - tcx) & 1)) * a.HC + ((N - 1 - tcx) >> 1);
                    const float a0 = wa[(ta * N + tcx) * a.WS], a1 = wa[(ta * N + tcx) * a.WS + 32];
                    float bv[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) bv[t] = tc[toff[t] + off];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        acc[0][t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, bv[t], acc[0][t], 0, 0, 0);
                        acc[1][t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, bv[t], acc[1][t], 0, 0, 0);
                    }
                }
        }
    }

    // accumulator register i of a tile: channel 8*(i/4) + 4*kk + (i%4) of its 32, MFMA column l32;
    // slice ks of the output-channel sum writes the ks-th copy of dx
    const int j = j0 + lj;
    dx += (size_t)ks * g.B * g.Cin * g.H * g.W;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int tr = (wpx * 4 + t) * subRows + lsub;
        const int b = b0 + (tr >> a.logTI), i = i0 + (tr & (a.TI - 1));
        if (b >= g.B || i >= g.H || j >= g.W) continue;
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ci = ci0 + wm * 64 + mi * 32 + 8 * (r / 4) + 4 * kk + (r % 4);
                if (ci < g.Cin) dx[(((size_t)b * g.Cin + ci) * g.H + i) * g.W + j] = acc[mi][t][r];
            }
    }
}

// dw[i] = sum over the partial copies, in an order that depends on (copies, R) only: the block's
// 256 threads are 256/R elements x R lanes, lane r adds copies r, r+R, r+2R, ... into four running
// sums taken in turn, and the R lane sums are added pairwise in a fixed tree.  R > 1 serves layers with few kernel
// elements and many copies.
__global__ __launch_bounds__(256) void ukst_sum_partials_kernel(const float* __restrict__ part,
                                                               float* __restrict__ dw, int n, int copies,
                                                               int logR)
{
    __shared__ float red[256];
    const int R = 1 << logR;
    const int r = threadIdx.x & (R - 1);
    const int i = blockIdx.x * (256 >> logR) + (threadIdx.x >> logR);
    // four running sums per lane (copies k, k+R, k+2R, k+3R in turn): four loads in flight
    float s = 0.f;
    if (i < n) {
        float s4[4] = {0.f, 0.f, 0.f, 0.f};
        int k = r;
        for (; k + 3 * R < copies; k += 4 * R) {
#pragma unroll
            for (int u = 0; u < 4; ++u) s4[u] += part[(size_t)(k + u * R) * n + i];
        }
        for (int u = 0; k < copies; k += R, ++u) s4[u] += part[(size_t)k * n + i];
        s = (s4[0] + s4[1]) + (s4[2] + s4[3]);
    }
    red[threadIdx.x] = s;
    for (int m = R >> 1; m > 0; m >>= 1) {
        __syncthreads();
        if (r < m) red[threadIdx.x] += red[threadIdx.x + m];
    }
    if (r == 0 && i < n) dw[i] = red[threadIdx.x];
}

// ------------------------------------------------------------------------------------------
// The same input gradient for bf16 operands on the bf16 matrix pipe: v_mfma_f32_32x32x8_bf16_1k
// takes 8 output channels per instruction, a lane holding four consecutive ones of its row or
// column.  LDS therefore keeps 8-byte elements of four output channels: weights packed once per
// call as [co/8][co%8/4][tap][ci][co%4], the dy tile transposed on its way in (a thread loads four
// columns of four channels and writes four elements), parity-split as before.
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

__global__ __launch_bounds__(256) void ukst_pack_w_bf16_kernel(const uint16_t* __restrict__ w,
                                                              uint16_t* __restrict__ wp, int Cout, int Cin,
                                                              int NN, int CoutP, int CIp)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;  // over [CoutP/4][NN][CIp][4]
    if (idx >= (size_t)CoutP * NN * CIp) return;
    const int q = (int)(idx & 3);
    const size_t r1 = idx >> 2;
    const int ci = (int)(r1 % CIp);
    const size_t r2 = r1 / CIp;
    const int tap = (int)(r2 % NN), co = (int)(r2 / NN) * 4 + q;
    wp[idx] = (co < Cout && ci < Cin) ? w[((size_t)co * Cin + ci) * NN + tap] : (uint16_t)0;
}

// SHIFT: how quads that straddle an end of their dy row are fetched.  false: element by element
// (best when most tiles lie inside the rows); true: one vector load from the nearest position
// inside the row, shifted into place (best for narrow maps, where every tile touches both ends:
// the batch then holds a single kind of load and waits once).
template <int N, bool SHIFT>
__global__ __launch_bounds__(256, 2) void ukst_grad_input_mfma_bf16_kernel(const uint16_t* __restrict__ dy,
                                                                          const uint16_t* __restrict__ wp,
                                                                          float* __restrict__ dx, GiMfmaArgs a)
{
    constexpr int NN = N * N;
    extern __shared__ __align__(16) u32x2 lds8[];
    const GeomBase& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kk = lane >> 5;
    const int wm = wave & (a.WM - 1), wpx = wave >> a.logWM;
    const int wlEls = NN * a.WS;                         // 8-byte elements per group of 4 channels
    const int tileEls = a.TB * a.LR * 2 * a.HC;
    u32x2* wl = lds8;                                    // [2][NN][WS]
    u32x2* tile = lds8 + 2 * wlEls;                      // [2][TB][LR][2][HC]

    const int lin = xcd_contiguous(blockIdx.y * gridDim.x + blockIdx.x, gridDim.x * gridDim.y);
    const int ks = lin / gridDim.x;
    int bid = lin - ks * gridDim.x;
    const int cit = bid % a.ciTiles; bid /= a.ciTiles;
    const int tx = bid % a.tilesX; bid /= a.tilesX;
    const int ty = bid % a.tilesY; bid /= a.tilesY;
    const int tb = bid;
    const int ci0 = cit * a.CI_T, i0 = ty * a.TI, j0 = tx * a.TJ, b0 = tb * a.TB;
    const int oy_base = 2 * i0 + g.P - (N - 1), ox_base = 2 * j0 + g.P - (N - 1);

    const int lj = l32 & (a.TJ - 1), lsub = l32 >> a.logTJ, subRows = 32 >> a.logTJ;
    int toff[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int tr = (wpx * 4 + t) * subRows + lsub;
        const int bl = tr >> a.logTI, li = tr & (a.TI - 1);
        toff[t] = kk * tileEls + ((bl * a.LR + 2 * li) * 2) * a.HC + lj;
    }
    const int a_base = kk * wlEls + wm * 64 + l32;
    f32x16 acc[2][4];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][t][i] = 0.f;

    const int rowsPerCo = a.TB * a.LR, cols = 2 * a.HC;
    const int c2n = 1 << a.logC4;  // 16-byte pieces per weight row (two elements each)
    const size_t plane = (size_t)g.OH * g.OW;
    const int co_begin = ks * a.coPer;
    const int co_end = co_begin + a.coPer < a.CoutP ? co_begin + a.coPer : a.CoutP;
    for (int co0 = co_begin; co0 < co_end; co0 += 8) {
        if (co0 != co_begin) __syncthreads();
        // packed weights of the round: eight 16-byte pieces in flight per thread; no predicates
        // (a written-out loop waits for every load): indices past the end repeat the last piece
        {
            const int npc = 2 * NN * c2n;
            for (int e0 = tid; e0 < npc; e0 += 256 * 8) {
                uint4 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = e0 + 256 * u < npc ? e0 + 256 * u : npc - 1;
                    v[u] = *reinterpret_cast<const uint4*>(
                        wp + (((size_t)(co0 >> 2) * NN + (e >> a.logC4)) * a.CIp + ci0 + 2 * (e & (c2n - 1))) * 4);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = e0 + 256 * u < npc ? e0 + 256 * u : npc - 1;
                    *reinterpret_cast<uint4*>(wl + (e >> a.logC4) * a.WS + 2 * (e & (c2n - 1))) = v[u];
                }
            }
        }
        // dy: task = (channel group of four, tile row, four columns)
        const int ntask = 2 * rowsPerCo * a.cols4;
        for (int e0 = tid; e0 < ntask; e0 += 256 * 4) {
            u32x2 q[4][4];
            int dst[4], ncol[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = e0 + 256 * u;
                dst[u] = -1;
#pragma unroll
                for (int c = 0; c < 4; ++c) q[u][c] = u32x2{0u, 0u};
                if (e < ntask) {
                    const int row = fdiv(e, a.dC4), cc = 4 * (e - row * a.cols4);
                    const int kg = fdiv(row, a.dRowsPerCo), rem = row - kg * rowsPerCo;
                    const int bl = fdiv(rem, a.dLR), rr = rem - bl * a.LR;
                    const int b = b0 + bl, oy = oy_base + rr, ox = ox_base + cc;
                    dst[u] = kg * tileEls + rem * cols + (cc >> 1);
                    ncol[u] = cols - cc;
                    if constexpr (SHIFT) {
                        if (b < g.B && oy >= 0 && oy < g.OH && ox + 3 >= 0 && ox < g.OW) {
                            const int cbase = co0 + 4 * kg;
                            const int start = ox < 0 ? 0 : (ox + 4 > g.OW ? g.OW - 4 : ox);
                            const int sh = 16 * (ox - start);  // > 0: drop leading elements
                            const size_t src = (((size_t)b * g.Cout + cbase) * g.OH + oy) * g.OW + start;
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                if (cbase + c >= g.Cout) continue;
                                typedef unsigned u2u __attribute__((ext_vector_type(2), aligned(2)));
                                const u2u t2 = *reinterpret_cast<const u2u*>(dy + src + c * plane);
                                unsigned long long v = ((unsigned long long)t2[1] << 32) | t2[0];
                                v = sh >= 0 ? v >> sh : v << -sh;  // whole elements, zeros moving in
                                q[u][c] = u32x2{(unsigned)v, (unsigned)(v >> 32)};
                            }
                        }
                    } else if (b < g.B && oy >= 0 && oy < g.OH && ox + 3 >= 0 && ox < g.OW) {
                        const int cbase = co0 + 4 * kg;
                        const size_t src = (((size_t)b * g.Cout + cbase) * g.OH + oy) * g.OW;
                        const bool whole = ox >= 0 && ox + 3 < g.OW;
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            if (cbase + c >= g.Cout) continue;
                            const uint16_t* pc = dy + src + c * plane;
                            if (whole) {
                                typedef unsigned u2u __attribute__((ext_vector_type(2), aligned(2)));
                                const u2u t2 = *reinterpret_cast<const u2u*>(pc + ox);
                                q[u][c] = u32x2{t2[0], t2[1]};
                            } else {
                                unsigned h[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                                for (int k = 0; k < 4; ++k)
                                    if (ox + k >= 0 && ox + k < g.OW) h[k] = pc[ox + k];
                                q[u][c] = u32x2{h[0] | (h[1] << 16), h[2] | (h[3] << 16)};
                            }
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (dst[u] >= 0) {
                    // element of column k: that column of channels 0..3
                    const unsigned lo = 0x05040100u, hi = 0x07060302u;
                    tile[dst[u]] = u32x2{__builtin_amdgcn_perm(q[u][1][0], q[u][0][0], lo),
                                         __builtin_amdgcn_perm(q[u][3][0], q[u][2][0], lo)};
                    tile[dst[u] + a.HC] = u32x2{__builtin_amdgcn_perm(q[u][1][0], q[u][0][0], hi),
                                                __builtin_amdgcn_perm(q[u][3][0], q[u][2][0], hi)};
                    if (ncol[u] > 2) {
                        tile[dst[u] + 1] = u32x2{__builtin_amdgcn_perm(q[u][1][1], q[u][0][1], lo),
                                                 __builtin_amdgcn_perm(q[u][3][1], q[u][2][1], lo)};
                        tile[dst[u] + a.HC + 1] = u32x2{__builtin_amdgcn_perm(q[u][1][1], q[u][0][1], hi),
                                                        __builtin_amdgcn_perm(q[u][3][1], q[u][2][1], hi)};
                    }
                }
        }
        __syncthreads();
        const u32x2* wa = wl + a_base;
#pragma unroll
        for (int ta = 0; ta < N; ++ta)
#pragma unroll
            for (int tcx = 0; tcx < N; ++tcx) {
                const int off = ((N - 1 - ta) * 2 + ((N - 1 - tcx) & 1)) * a.HC + ((N - 1 - tcx) >> 1);
                const s16x4 a0 = __builtin_bit_cast(s16x4, wa[(ta * N + tcx) * a.WS]);
                const s16x4 a1 = __builtin_bit_cast(s16x4, wa[(ta * N + tcx) * a.WS + 32]);
                s16x4 bv[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) bv[t] = __builtin_bit_cast(s16x4, tile[toff[t] + off]);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    acc[0][t] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a0, bv[t], acc[0][t], 0, 0, 0);
                    acc[1][t] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a1, bv[t], acc[1][t], 0, 0, 0);
                }
            }
    }

    const int j = j0 + lj;
    dx += (size_t)ks * g.B * g.Cin * g.H * g.W;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int tr = (wpx * 4 + t) * subRows + lsub;
        const int b = b0 + (tr >> a.logTI), i = i0 + (tr & (a.TI - 1));
        if (b >= g.B || i >= g.H || j >= g.W) continue;
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ci = ci0 + wm * 64 + mi * 32 + 8 * (r / 4) + 4 * kk + (r % 4);
                if (ci < g.Cin) dx[(((size_t)b * g.Cin + ci) * g.H + i) * g.W + j] = acc[mi][t][r];
            }
    }
}

// Fills the launch description; false if this shape is better served by the vector-ALU kernel.
// packed16: the description of the bf16 kernel (8-byte LDS elements of four channels, rounds of 8)
bool gi_mfma_args(const Geom& g, GiMfmaArgs& a, bool packed16 = false)
{
    if (g.Cin < 32 || g.Cout < 16) return false;
    const int N = g.n, NN = N * N;
    for (int WM = (g.Cin > 64 ? 2 : 1); WM >= 1; --WM) {
        a.g = g;
        a.WM = WM; a.logWM = WM == 2 ? 1 : 0;
        a.CI_T = 64 * WM; a.logC4 = (WM == 2 ? 5 : 4) + (packed16 ? 1 : 0);
        a.WS = a.CI_T + (packed16 ? 2 : 4);
        a.TJ = pow2_ceil(g.W < 32 ? g.W : 32);
        if (a.TJ < 4) a.TJ = 4;
        a.logTJ = log2_of(a.TJ);
        const int TR = (16 / WM) * (32 / a.TJ);  // 4 MFMA row groups per wave, 4 / WM waves along them
        a.TI = pow2_ceil(g.H < TR ? g.H : TR);
        a.TB = TR / a.TI;
        a.logTI = log2_of(a.TI);
        a.LR = 2 * a.TI + N - 2;
        a.HC = a.TJ + N / 2;
        const size_t perCo = (size_t)4 * (NN * a.WS + a.TB * a.LR * 2 * a.HC);
        int cc = (int)((76 * 1024) / perCo) & ~1;
        if (cc > 8) cc = 8;
        if (packed16) cc = (size_t)16 * (NN * a.WS + a.TB * a.LR * 2 * a.HC) <= 76 * 1024 ? 8 : 0;
        if (cc < 2) continue;
        a.CC = cc;
        a.CoutP = (g.Cout + cc - 1) / cc * cc;
        a.CIp = (g.Cin + a.CI_T - 1) / a.CI_T * a.CI_T;
        a.tilesX = (g.W + a.TJ - 1) / a.TJ;
        a.tilesY = (g.H + a.TI - 1) / a.TI;
        a.tilesB = (g.B + a.TB - 1) / a.TB;
        a.ciTiles = a.CIp / a.CI_T;
        a.cols4 = (2 * a.HC + 3) / 4;
        a.dC4 = make_fastdiv((unsigned)a.cols4);
        a.dRowsPerCo = make_fastdiv((unsigned)(a.TB * a.LR));
        a.dLR = make_fastdiv((unsigned)a.LR);
        const long long nb = (long long)a.tilesX * a.tilesY * a.tilesB * a.ciTiles;
        if (nb > 0x7fffffffLL) return false;
        if ((size_t)a.CoutP * NN * a.CIp > 0x7fffffffu) return false;
        // few tiles: split the sum over output channels into slices (one copy of dx each, added in
        // a fixed order afterwards) until the grid has two blocks per compute unit
        int ks = 1;
        const int rounds = a.CoutP / cc;
        while (nb * ks < 512 && ks * 2 <= rounds && ks < 32) ks *= 2;
        a.coPer = (rounds + ks - 1) / ks * cc;
        a.KS = (a.CoutP + a.coPer - 1) / a.coPer;
        if (a.KS > 1 && (size_t)g.B * g.Cin * g.H * g.W > 0x7fffffffu) { a.KS = 1; a.coPer = a.CoutP; }
        return true;
    }
    return false;
}

template <int N>
hipError_t launch_gi_mfma_bf16(const GiMfmaArgs& a, const void* dy, const void* w, float* dx, Workspace& ws,
                               hipStream_t stream)
{
    const GeomBase& g = a.g;
    const size_t pelems = (size_t)a.CoutP * N * N * a.CIp;           // bf16 elements
    const size_t pbytes = ws_align(pelems * 2);
    const size_t xelems = (size_t)g.B * g.Cin * g.H * g.W;
    // workspace: packed weights, then (split sums) the copies of dx
    const size_t need = pbytes + (a.KS > 1 ? xelems * a.KS * 4 : 0);
    if (ws.query) { ws.need = need; return hipSuccess; }
    if (ws.bytes < need) return kWorkspaceTooSmall;
    unsigned char* scratch = (unsigned char*)ws.ptr;
    hipError_t e;
    uint16_t* wp = (uint16_t*)scratch;
    float* part = (float*)(scratch + pbytes);
    hipLaunchKernelGGL(ukst_pack_w_bf16_kernel, dim3((unsigned)((pelems + 255) / 256)), dim3(256), 0, stream,
                       (const uint16_t*)w, wp, g.Cout, g.Cin, N * N, a.CoutP, a.CIp);
    e = hipGetLastError();
    if (e == hipSuccess) {
        const size_t lds = (size_t)16 * (N * N * a.WS + a.TB * a.LR * 2 * a.HC);
        // maps of at most 16 columns (every tile touches both ends of the dy rows, which must hold
        // a whole quad) take the shifting variant
        const bool shift = g.W <= 16 && g.OW >= 4;
        typedef void (*kernel_t)(const uint16_t*, const uint16_t*, float*, GiMfmaArgs);
        const kernel_t kfn = shift ? ukst_grad_input_mfma_bf16_kernel<N, true>
                                   : ukst_grad_input_mfma_bf16_kernel<N, false>;
        e = hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e == hipSuccess) {
            const unsigned nb = (unsigned)((long long)a.tilesX * a.tilesY * a.tilesB * a.ciTiles);
            hipLaunchKernelGGL(kfn, dim3(nb, (unsigned)a.KS), dim3(256), lds, stream, (const uint16_t*)dy,
                               (const uint16_t*)wp, a.KS > 1 ? part : dx, a);
            e = hipGetLastError();
        }
        if (e == hipSuccess && a.KS > 1) {
            hipLaunchKernelGGL(ukst_sum_partials_kernel, dim3((unsigned)((xelems + 255) / 256)), dim3(256), 0,
                               stream, (const float*)part, dx, (int)xelems, a.KS, 0);
            e = hipGetLastError();
        }
    }
    return e;
}

template <int N, typename TIn>
hipError_t launch_gi_mfma(const GiMfmaArgs& a, const void* dy, const void* w, float* dx, Workspace& ws,
                          hipStream_t stream)
{
    const GeomBase& g = a.g;
    const size_t pelems = (size_t)a.CoutP * N * N * a.CIp;
    const size_t xelems = (size_t)g.B * g.Cin * g.H * g.W;
    // workspace: packed weights, then (split sums) the copies of dx
    const size_t need = (pelems + (a.KS > 1 ? xelems * a.KS : 0)) * sizeof(float);
    if (ws.query) { ws.need = need; return hipSuccess; }
    if (ws.bytes < need) return kWorkspaceTooSmall;
    float* wp = (float*)ws.ptr;
    hipError_t e;
    float* part = wp + pelems;
    hipLaunchKernelGGL((ukst_pack_w_kernel<TIn>), dim3((unsigned)((pelems + 255) / 256)), dim3(256), 0, stream,
                       (const TIn*)w, wp, g.Cout, g.Cin, N * N, a.CoutP, a.CIp);
    e = hipGetLastError();
    if (e == hipSuccess) {
        const size_t lds = (size_t)4 * a.CC * (N * N * a.WS + a.TB * a.LR * 2 * a.HC);
        const void* kfn = (const void*)ukst_grad_input_mfma_kernel<N, TIn>;
        e = hipFuncSetAttribute(kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e == hipSuccess) {
            const unsigned nb = (unsigned)((long long)a.tilesX * a.tilesY * a.tilesB * a.ciTiles);
            hipLaunchKernelGGL((ukst_grad_input_mfma_kernel<N, TIn>), dim3(nb, (unsigned)a.KS), dim3(256), lds,
                               stream, (const TIn*)dy, (const float*)wp, a.KS > 1 ? part : dx, a);
            e = hipGetLastError();
        }
        if (e == hipSuccess && a.KS > 1) {
            hipLaunchKernelGGL(ukst_sum_partials_kernel, dim3((unsigned)((xelems + 255) / 256)), dim3(256), 0,
                               stream, (const float*)part, dx, (int)xelems, a.KS, 0);
            e = hipGetLastError();
        }
    }
    return e;
}

// Block count of a (CI_BLK, PX) choice: the widest register block that still gives the chip two
// blocks per compute unit wins; small maps with many channels fall back to narrower blocks.
long long gi_blocks(const Geom& g, int ci_blk, int px)
{
    int TJ = pow2_ceil(g.W < 32 ? g.W : 32);
    if (TJ < 4) TJ = 4;
    const int TR = px * 256 / TJ;
    const int TI = pow2_ceil(g.H < TR ? g.H : TR), TB = TR / TI;
    return (long long)((g.W + TJ - 1) / TJ) * ((g.H + TI - 1) / TI) * ((g.B + TB - 1) / TB) *
           ((g.Cin + ci_blk - 1) / ci_blk);
}

template <int N, typename TIn>
hipError_t launch_gi_t(const Geom& g, const void* dy, const void* w, float* dx, hipStream_t stream)
{
    if (g.Cin <= 4) return launch_gi<N, 4, 2, TIn>(g, dy, w, dx, stream);
    if (g.Cin <= 8) return launch_gi<N, 8, 1, TIn>(g, dy, w, dx, stream);
    if (gi_blocks(g, 16, 2) >= 512) return launch_gi<N, 16, 2, TIn>(g, dy, w, dx, stream);
    if (gi_blocks(g, 16, 1) >= 512) return launch_gi<N, 16, 1, TIn>(g, dy, w, dx, stream);
    return launch_gi<N, 8, 1, TIn>(g, dy, w, dx, stream);
}

template <int N>
hipError_t launch_gi_n(const Geom& g, const void* dy, const void* w, float* dx, int dtype,
                       Workspace& ws, hipStream_t stream)
{
    if (grad_input_window_supported(g, dtype)) return launch_grad_input_window(g, dy, w, dx, ws, stream);
    if (grad_narrow_supported(g, dtype)) return launch_grad_narrow(0, g, dy, w, dx, ws, stream);
    GiMfmaArgs ma;
    if (dtype == 1 && gi_mfma_args(g, ma, true)) return launch_gi_mfma_bf16<N>(ma, dy, w, dx, ws, stream);
    if (gi_mfma_args(g, ma))
        return dtype == 1 ? launch_gi_mfma<N, uint16_t>(ma, dy, w, dx, ws, stream)
                          : launch_gi_mfma<N, float>(ma, dy, w, dx, ws, stream);
    if (ws.query) return hipSuccess;  // the vector-ALU kernel uses no scratch
    return dtype == 1 ? launch_gi_t<N, uint16_t>(g, dy, w, dx, stream)
                      : launch_gi_t<N, float>(g, dy, w, dx, stream);
}

// ------------------------------------------------------------------------------------------
// Gradient with respect to the kernel.
//
// A reduction over batch and space with a small result.  Block = TP x TCO x TCI threads: a thread
// owns CO_R x CI_R (output, input) channel pairs for all n*n taps and every TP-th pixel of the
// staged tile (TI x TJ input pixels of one image with the dy rows above them); wide layers use
// TP = 1 and 16 x 16 channel threads, narrow layers put all 256 threads on pixels.  A block walks
// over a slice of the tiles; lanes that differ only in their pixel share are summed with wave
// shuffles, and every (slice, wave group) writes its partial result to its own copy of dw, which
// ukst_sum_partials_kernel adds in a fixed order (bit-reproducible, no atomics).
struct GradWArgs {
    GeomBase g;
    int TCO, TCI, PB, TP;      // threads along co, ci; PB = TCO*TCI; TP = 256 / PB
    int logTCI, logPB;
    int TI, TJ, logTJ;         // staged pixel tile
    int LR, LC;                // staged dy rows / columns
    int XS;                    // floats per staged pixel (CI_T + pad)
    int tilesX, tilesY, nStages, stagesPerSlice, nSlices;
    int coTiles, ciTiles;
    int SUB;                   // partial copies a block writes (wave groups that share pairs)
    int LC4;                   // four-column pieces per staged dy row
    int foldWaves;             // 1: the block adds its four waves' sums in LDS and writes one copy
    FastDiv dLC4, dLR;
};

template <int N, int CO_R, int CI_R, typename TIn>
__global__ __launch_bounds__(256) void ukst_grad_weight_kernel(const TIn* __restrict__ x,
                                                              const TIn* __restrict__ dy,
                                                              float* __restrict__ part, GradWArgs a)
{
    constexpr int NN = N * N;
    extern __shared__ __align__(16) float lds_f[];
    const GeomBase& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int CO_T = a.TCO * CO_R, CI_T = a.TCI * CI_R;
    float* xs = lds_f;                               // [TI*TJ][XS]
    float* dys = lds_f + a.TI * a.TJ * a.XS;         // [CO_T][LR][LC]

    int bid = xcd_contiguous(blockIdx.x, gridDim.x);  // neighbours in this numbering share an L2
    const int cit = bid % a.ciTiles; bid /= a.ciTiles;
    const int cot = bid % a.coTiles; bid /= a.coTiles;
    const int slice = bid;
    const int co0 = cot * CO_T, ci0 = cit * CI_T;

    const int q = tid & (a.PB - 1), tp = tid >> a.logPB;
    const int tci = q & (a.TCI - 1), tco = q >> a.logTCI;

    float acc[CO_R][CI_R][NN];
#pragma unroll
    for (int c = 0; c < CO_R; ++c)
#pragma unroll
        for (int k = 0; k < CI_R; ++k)
#pragma unroll
            for (int t = 0; t < NN; ++t) acc[c][k][t] = 0.f;

    const int st_end = (slice + 1) * a.stagesPerSlice < a.nStages ? (slice + 1) * a.stagesPerSlice : a.nStages;
    const int npix = a.TI * a.TJ, planeLR = a.LR * a.LC;
    for (int st = slice * a.stagesPerSlice; st < st_end; ++st) {
        int t = st;
        const int tx = t % a.tilesX; t /= a.tilesX;
        const int ty = t % a.tilesY; t /= a.tilesY;
        const int b = t;
        const int i0 = ty * a.TI, j0 = tx * a.TJ;
        const int oy_base = 2 * i0 + g.P - (N - 1), ox_base = 2 * j0 + g.P - (N - 1);
        __syncthreads();
        // x tile: xs[pixel][channel], lanes along the pixel row (coalesced reads)
        // x tile as xs[pixel][channel] and the dy rows above it as dys[channel][row][column]; a
        // thread moves four consecutive pixels / columns with one vector load (scalar loads where
        // they straddle the end of a row), everything outside the tensors becomes zeros
        {
            const int nq = a.TJ >= 4 ? (CI_T * npix) >> 2 : 0;
            for (int e0 = tid; e0 < nq; e0 += 256 * 4) {
                Quad q[4];
                int dst[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int e = e0 + 256 * u;
                    dst[u] = -1;
                    q[u] = Quad{{0.f, 0.f, 0.f, 0.f}};
                    if (e < nq) {
                        const int p = (e << 2) & (npix - 1), cl = (e << 2) / npix;
                        const int li = p >> a.logTJ, ljx = p & (a.TJ - 1);
                        const int i = i0 + li, j = j0 + ljx, ci = ci0 + cl;
                        dst[u] = p * a.XS + cl;
                        if (ci < g.Cin && i < g.H && j < g.W) {
                            const size_t src = (((size_t)b * g.Cin + ci) * g.H + i) * g.W;
                            if (j + 3 < g.W) {
                                q[u] = ld_quad(x, src + j);
                            } else {
#pragma unroll
                                for (int k = 0; k < 4; ++k)
                                    if (j + k < g.W) q[u].v[k] = ld_f32(x, src + j + k);
                            }
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (dst[u] >= 0) {
#pragma unroll
                        for (int k = 0; k < 4; ++k) xs[dst[u] + k * a.XS] = q[u].v[k];
                    }
            }
            if (a.TJ < 4)
                stage_elements<8>(xs, tid, CI_T * npix, [&](int e, int& dst) {
                    const int p = e & (npix - 1), cl = e / npix;
                    const int li = p >> a.logTJ, ljx = p & (a.TJ - 1);
                    const int i = i0 + li, j = j0 + ljx, ci = ci0 + cl;
                    dst = p * a.XS + cl;
                    return (ci < g.Cin && i < g.H && j < g.W)
                               ? ld_f32(x, (((size_t)b * g.Cin + ci) * g.H + i) * g.W + j) : 0.f;
                });
            const int nd = CO_T * a.LR * a.LC4;
            for (int e0 = tid; e0 < nd; e0 += 256 * 10) {
                Quad q[10];
                int dst[10], ncol[10];
#pragma unroll
                for (int u = 0; u < 10; ++u) {
                    const int e = e0 + 256 * u;
                    dst[u] = -1;
                    q[u] = Quad{{0.f, 0.f, 0.f, 0.f}};
                    if (e < nd) {
                        const int row = fdiv(e, a.dLC4), cc = 4 * (e - row * a.LC4);
                        const int col = fdiv(row, a.dLR), rr = row - col * a.LR;
                        const int co = co0 + col, oy = oy_base + rr, ox = ox_base + cc;
                        dst[u] = row * a.LC + cc;
                        ncol[u] = a.LC - cc;
                        if (co < g.Cout && oy >= 0 && oy < g.OH && ox + 3 >= 0 && ox < g.OW) {
                            const size_t src = (((size_t)b * g.Cout + co) * g.OH + oy) * g.OW;
                            if (ox >= 0 && ox + 3 < g.OW) {
                                q[u] = ld_quad(dy, src + ox);
                            } else {
#pragma unroll
                                for (int k = 0; k < 4; ++k)
                                    if (ox + k >= 0 && ox + k < g.OW) q[u].v[k] = ld_f32(dy, src + ox + k);
                            }
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < 10; ++u)
                    if (dst[u] >= 0) {
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (k < ncol[u]) dys[dst[u] + k] = q[u].v[k];
                    }
            }
        }
        __syncthreads();
        for (int p = tp; p < npix; p += a.TP) {
            const int li = p >> a.logTJ, ljx = p & (a.TJ - 1);
            float xv[CI_R];
            const float* xp = xs + p * a.XS + tci * CI_R;
            if constexpr (CI_R % 4 == 0) {
#pragma unroll
                for (int k = 0; k < CI_R; k += 4) {
                    const float4 t4 = *reinterpret_cast<const float4*>(xp + k);
                    xv[k] = t4.x; xv[k + 1] = t4.y; xv[k + 2] = t4.z; xv[k + 3] = t4.w;
                }
            } else {
#pragma unroll
                for (int k = 0; k < CI_R; ++k) xv[k] = xp[k];
            }
            const float* dp = dys + (tco * CO_R) * planeLR + (2 * li) * a.LC + 2 * ljx;
#pragma unroll
            for (int c = 0; c < CO_R; ++c)
#pragma unroll
                for (int ta = 0; ta < N; ++ta)
#pragma unroll
                    for (int tcx = 0; tcx < N; ++tcx) {
                        const float d = dp[c * planeLR + (N - 1 - ta) * a.LC + (N - 1 - tcx)];
#pragma unroll
                        for (int k = 0; k < CI_R; ++k)
                            acc[c][k][ta * N + tcx] = fmaf(d, xv[k], acc[c][k][ta * N + tcx]);
                    }
        }
    }

    // lanes of a wave that hold the same channel pairs (they differ in tp only) are summed
    for (int m = a.PB; m < 64; m <<= 1)
#pragma unroll
        for (int c = 0; c < CO_R; ++c)
#pragma unroll
            for (int k = 0; k < CI_R; ++k)
#pragma unroll
                for (int t = 0; t < NN; ++t) acc[c][k][t] += __shfl_xor(acc[c][k][t], m, 64);
    int sub = tid >> (a.logPB > 6 ? a.logPB : 6);  // wave group: waves that share pairs differ in it
    if (a.foldWaves) {
        // few pairs and few taps: the four waves' sums meet in LDS (fixed order) and the block
        // writes one copy instead of four
        constexpr int R = CO_R * CI_R * NN;
        __syncthreads();  // the staged tiles are no longer read
        if (lane < a.PB) {
            float* r = lds_f + ((tid >> 6) * a.PB + lane) * R;
#pragma unroll
            for (int c = 0; c < CO_R; ++c)
#pragma unroll
                for (int k = 0; k < CI_R; ++k)
#pragma unroll
                    for (int t = 0; t < NN; ++t) r[(c * CI_R + k) * NN + t] = acc[c][k][t];
        }
        __syncthreads();
        if (tid >= a.PB) return;
#pragma unroll
        for (int c = 0; c < CO_R; ++c)
#pragma unroll
            for (int k = 0; k < CI_R; ++k)
#pragma unroll
                for (int t = 0; t < NN; ++t) {
                    const int i = (c * CI_R + k) * NN + t;
                    acc[c][k][t] = ((lds_f[tid * R + i] + lds_f[(a.PB + tid) * R + i]) +
                                    lds_f[(2 * a.PB + tid) * R + i]) + lds_f[(3 * a.PB + tid) * R + i];
                }
        sub = 0;
    } else if (a.PB < 64 && lane >= a.PB) {
        return;
    }
    float* out = part + (size_t)(slice * a.SUB + sub) * g.Cout * g.Cin * NN;
#pragma unroll
    for (int c = 0; c < CO_R; ++c) {
        const int co = co0 + tco * CO_R + c;
        if (co >= g.Cout) continue;
#pragma unroll
        for (int k = 0; k < CI_R; ++k) {
            const int ci = ci0 + tci * CI_R + k;
            if (ci >= g.Cin) continue;
#pragma unroll
            for (int t = 0; t < NN; ++t) out[((size_t)co * g.Cin + ci) * NN + t] = acc[c][k][t];
        }
    }
}

// ------------------------------------------------------------------------------------------
// Gradient with respect to the kernel on the matrix cores (wide layers, either dtype).
//
// Per tap the reduction is a dense product over pixels: DW_tap[co][ci] += sum_pixel
// DY_tap[co][pixel] * X[ci][pixel].  v_mfma_f32_32x32x2_f32 takes 32 output channels x 32 input
// channels x two neighbouring pixels per instruction.  The n*n taps of a block's 32 x (32*NC)
// channel tile are dealt to its four waves (tap t belongs to wave t % 4), so a wave keeps
// ceil(n*n/4) * NC accumulator tiles and every x fragment it reads feeds all of its taps.  The
// staged tile is TR (image, pixel row) pairs x TJ pixel columns with the dy rows above them,
// parity-split as in the other kernels so that a tap's lattice is contiguous; per-channel strides
// are odd so that the 32 channels of a fragment fall into 32 banks.  Blocks walk over slices of
// the tiles and write partial results as [slice][co][tap][ci] (lanes along ci);
// ukst_sum_taps_kernel adds the slices in a fixed order and stores dw[co][ci][tap].
typedef __bf16 gw_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 gw_bf16x8u __attribute__((ext_vector_type(8), aligned(2)));
typedef unsigned gw_u4 __attribute__((ext_vector_type(4)));
typedef unsigned gw_u4u __attribute__((ext_vector_type(4), aligned(2)));
typedef unsigned gw_u2 __attribute__((ext_vector_type(2)));
constexpr unsigned kGwInvalid = 0xFFFFFF00u;  // byte offset that is out of range for any buffer
constexpr int kGwRsrcFlags = 0x00020000;      // raw 32-bit buffer, gfx9 family


struct GwMfmaArgs {
    GeomBase g;
    int TJ, logTJ, TI, logTI, TB, TR, logPix;  // logPix = log2(TR * TJ)
    int LR, HC, cols, DP, XP;
    int tilesX, tilesY, nStages, stagesPerSlice, nSlices;
    int coTiles, ciTiles;
    int cols4;                 // four-column pieces per staged dy row
    int fast, npass;           // piecewise staging (rows of at least four elements), its passes per channel
    FastDiv dC4, dRows, dLR;
};

template <int N, int NC, typename TIn>
__global__ __launch_bounds__(256, 2) void ukst_grad_weight_mfma_kernel(const TIn* __restrict__ x,
                                                                      const TIn* __restrict__ dy,
                                                                      float* __restrict__ part, GwMfmaArgs a)
{
    constexpr int NN = N * N, TS = (NN + 3) / 4, CI_T = 32 * NC;
    extern __shared__ __align__(16) float lds_f[];
    const GeomBase& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kk = lane >> 5;
    float* xs = lds_f;                     // [CI_T][XP]
    float* dys = lds_f + CI_T * a.XP;      // [32][DP]
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
        (void*)x, 0, (int)((size_t)g.B * g.Cin * g.H * g.W * sizeof(TIn)), kGwRsrcFlags);
    const __amdgpu_buffer_rsrc_t rs_dy = __builtin_amdgcn_make_buffer_rsrc(
        (void*)dy, 0, (int)((size_t)g.B * g.Cout * g.OH * g.OW * sizeof(TIn)), kGwRsrcFlags);

    int bid = xcd_contiguous(blockIdx.x, gridDim.x);  // neighbours in this numbering share an L2
    const int cit = bid % a.ciTiles; bid /= a.ciTiles;
    const int cot = bid % a.coTiles; bid /= a.coTiles;
    const int slice = bid;
    const int co0 = cot * 32, ci0 = cit * CI_T;

    const int nts = (NN - wave + 3) / 4;   // taps of this wave: wave, wave + 4, ...
    int tapoff[TS];
#pragma unroll
    for (int ts = 0; ts < TS; ++ts) {
        const int t = wave + 4 * ts < NN ? wave + 4 * ts : 0;
        const int ta = t / N, tc = t % N;
        tapoff[ts] = (N - 1 - ta) * a.cols + ((N - 1 - tc) & 1) * a.HC + ((N - 1 - tc) >> 1);
    }
    f32x16 acc[TS][NC];
#pragma unroll
    for (int ts = 0; ts < TS; ++ts)
#pragma unroll
        for (int nc = 0; nc < NC; ++nc)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ts][nc][i] = 0.f;

    const int npix = 1 << a.logPix, rowsPerCo = a.TB * a.LR;
    const int a_lane = l32 * a.DP + kk, b_lane = l32 * a.XP + kk;
    const int st_end = (slice + 1) * a.stagesPerSlice < a.nStages ? (slice + 1) * a.stagesPerSlice : a.nStages;
    for (int st = slice * a.stagesPerSlice; st < st_end; ++st) {
        int t = st;
        const int tx = t % a.tilesX; t /= a.tilesX;
        const int ty = t % a.tilesY; t /= a.tilesY;
        const int b0 = t * a.TB, i0 = ty * a.TI, j0 = tx * a.TJ;
        const int oy_base = 2 * i0 + g.P - (N - 1), ox_base = 2 * j0 + g.P - (N - 1);
        __syncthreads();
        if (a.fast) {
            // Staging without divergent address arithmetic per piece (pieces of four elements):
            // every wave owns a quarter of the channels; what depends on the lane (row, piece,
            // validity) is worked out once per stage and pass, the channel enters through the
            // scalar offset of a buffer load, and a group's loads are requested before the
            // previous group is written.  Rows, images and channels that do not exist are read
            // through an out-of-range offset and arrive as zeros; a piece that hangs over an end
            // of its row is fetched from inside the row and shifted into place.
            constexpr int ES = (int)sizeof(TIn);
            constexpr int GRP = 4;
            const int per_co = rowsPerCo * a.cols4;
            const unsigned co_bytes = (unsigned)(g.OH * g.OW * ES);
            unsigned dvoff;
            int dsh, ddst, dnc;
            auto lane_pass = [&](int pp) {
                const int idx = lane + 64 * pp;
                const int rem = fdiv(idx, a.dC4), m = idx - rem * a.cols4;
                const int bl = fdiv(rem, a.dLR), rr = rem - bl * a.LR;
                const int b = b0 + bl, oy = oy_base + rr, ox = ox_base + 4 * m;
                const bool ok = idx < per_co && b < g.B && oy >= 0 && oy < g.OH && ox + 3 >= 0 && ox < g.OW;
                const int oxl = ox < 0 ? 0 : (ox > g.OW - 4 ? g.OW - 4 : ox);
                dsh = oxl - ox;
                dvoff = ok ? (unsigned)((((b * g.Cout) * g.OH + oy) * g.OW + oxl) * ES) : kGwInvalid;
                ddst = idx < per_co ? rem * a.cols + 2 * m : -1;
                dnc = a.cols - 4 * m;  // columns of this piece that belong to the staged row (2 or >= 4)
            };
            auto load_piece = [&](const __amdgpu_buffer_rsrc_t& rs, unsigned voff, unsigned soff) -> Quad {
                if constexpr (ES == 4) {
                    const gw_u4 t = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soff, 0);
                    return Quad{{__uint_as_float(t.x), __uint_as_float(t.y), __uint_as_float(t.z), __uint_as_float(t.w)}};
                } else {
                    const gw_u2 t = __builtin_amdgcn_raw_buffer_load_b64(rs, voff, soff, 0);
                    return Quad{{__uint_as_float(t.x << 16), __uint_as_float(t.x & 0xFFFF0000u),
                                 __uint_as_float(t.y << 16), __uint_as_float(t.y & 0xFFFF0000u)}};
                }
            };
            // four elements moved sh places up (sh > 0) or down, zeros moving in; 0 < |sh| < 4
            auto shifted = [&](const Quad& q, int sh) -> Quad {
                Quad r;
#pragma unroll
                for (int k2 = 0; k2 < 4; ++k2) {
                    const int src = k2 - sh;
                    float v = 0.f;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v = src == e ? q.v[e] : v;
                    r.v[k2] = v;
                }
                return r;
            };
            auto load_group = [&](int h, Quad (&q)[GRP]) {
#pragma unroll
                for (int c4 = 0; c4 < GRP; ++c4) {
                    const int co = co0 + wave * 8 + h * GRP + c4;  // uniform
                    const bool cok = co < g.Cout;
                    q[c4] = load_piece(rs_dy, cok ? dvoff : kGwInvalid, cok ? (unsigned)co * co_bytes : 0u);
                }
            };
            auto write_group = [&](int h, int sh, int dst, int nc, const Quad (&q)[GRP]) {
                if (dst < 0) return;
#pragma unroll
                for (int c4 = 0; c4 < GRP; ++c4) {
                    float* base = dys + (wave * 8 + h * GRP + c4) * a.DP + dst;
                    const Quad v = sh != 0 ? shifted(q[c4], sh) : q[c4];
                    base[0] = v.v[0];
                    base[a.HC] = v.v[1];
                    if (nc > 2) {
                        base[1] = v.v[2];
                        base[a.HC + 1] = v.v[3];
                    }
                }
            };
            Quad qa[GRP], qb[GRP];
            lane_pass(0);
            load_group(0, qa);
            {
                // x tile: four pixels of a row per piece
                const int logCPC = a.logPix - 2, CPC = 1 << logCPC;  // pieces per channel
                const int cw0 = wave * (CI_T / 4);
                const int xpasses = ((CI_T / 4) << logCPC) >> 6;
                for (int p0 = 0; p0 < xpasses; p0 += 4) {
                    Quad q[4];
                    int dst[4], sh[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        dst[u] = -1;
                        sh[u] = 0;
                        if (p0 + u < xpasses) {
                            const int flat = lane + 64 * (p0 + u);
                            const int cl = cw0 + (flat >> logCPC), pix = (flat & (CPC - 1)) << 2;
                            const int tr = pix >> a.logTJ, lj = pix & (a.TJ - 1);
                            const int b = b0 + (tr >> a.logTI), i = i0 + (tr & (a.TI - 1)), j = j0 + lj, ci = ci0 + cl;
                            const bool ok = ci < g.Cin && b < g.B && i < g.H && j < g.W;
                            const int jl = j > g.W - 4 ? g.W - 4 : j;
                            sh[u] = jl - j;
                            const unsigned voff = ok ? (unsigned)((((b * g.Cin + ci) * g.H + i) * g.W + jl) * ES) : kGwInvalid;
                            q[u] = load_piece(rs_x, voff, 0u);
                            dst[u] = cl * a.XP + pix;
                        }
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (dst[u] >= 0) {
                            const Quad v = sh[u] != 0 ? shifted(q[u], sh[u]) : q[u];
#pragma unroll
                            for (int k2 = 0; k2 < 4; ++k2) xs[dst[u] + k2] = v.v[k2];
                        }
                }
            }
#pragma unroll 1
            for (int pp = 0; pp < a.npass; ++pp) {
                const int sh_c = dsh, dst_c = ddst, nc_c = dnc;
                load_group(1, qb);
                write_group(0, sh_c, dst_c, nc_c, qa);
                if (pp + 1 < a.npass) {
                    lane_pass(pp + 1);
                    load_group(0, qa);
                }
                write_group(1, sh_c, dst_c, nc_c, qb);
            }
        } else {
        if (a.logTJ >= 2) {
            // x tile, four pixels of a row per thread (one vector load unless they straddle the row end)
            const int nq = (CI_T * npix) >> 2;
            for (int e0 = tid; e0 < nq; e0 += 256 * 4) {
                Quad q[4];
                int dst[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int e = e0 + 256 * u;
                    dst[u] = -1;
                    q[u] = Quad{{0.f, 0.f, 0.f, 0.f}};
                    if (e < nq) {
                        const int pix = (e << 2) & (npix - 1), cl = (e << 2) >> a.logPix;
                        const int tr = pix >> a.logTJ, lj = pix & (a.TJ - 1);
                        const int b = b0 + (tr >> a.logTI), i = i0 + (tr & (a.TI - 1)), j = j0 + lj, ci = ci0 + cl;
                        dst[u] = cl * a.XP + pix;
                        if (ci < g.Cin && b < g.B && i < g.H && j < g.W) {
                            const size_t src = (((size_t)b * g.Cin + ci) * g.H + i) * g.W;
                            if (j + 3 < g.W) {
                                q[u] = ld_quad(x, src + j);
                            } else {
#pragma unroll
                                for (int k = 0; k < 4; ++k)
                                    if (j + k < g.W) q[u].v[k] = ld_f32(x, src + j + k);
                            }
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (dst[u] >= 0) {
#pragma unroll
                        for (int k = 0; k < 4; ++k) xs[dst[u] + k] = q[u].v[k];
                    }
            }
        } else
        stage_elements<8>(xs, tid, CI_T * npix, [&](int e, int& dst) {
            const int pix = e & (npix - 1), cl = e >> a.logPix;
            const int tr = pix >> a.logTJ, lj = pix & (a.TJ - 1);
            const int b = b0 + (tr >> a.logTI), i = i0 + (tr & (a.TI - 1)), j = j0 + lj, ci = ci0 + cl;
            dst = cl * a.XP + pix;
            return (ci < g.Cin && b < g.B && i < g.H && j < g.W)
                       ? ld_f32(x, (((size_t)b * g.Cin + ci) * g.H + i) * g.W + j) : 0.f;
        });
        {
            DyTile t;
            t.nrows = 32 * rowsPerCo; t.rowsPerCo = rowsPerCo; t.coStride = a.DP; t.cols = a.cols;
            t.cols4 = a.cols4; t.HC = a.HC; t.LR = a.LR; t.co_first = co0; t.co_end = g.Cout; t.b0 = b0;
            t.oy_base = oy_base; t.ox_base = ox_base; t.dC4 = a.dC4; t.dRowsPerCo = a.dRows; t.dLR = a.dLR;
            stage_dy_tile<8>(dys, dy, g, t, tid);
        }
        }
        __syncthreads();
        const int wj = g.W - j0 < a.TJ ? g.W - j0 : a.TJ;
        const int steps = (wj + 1) >> 1;
        // the tap count of a wave is TS or TS - 1: one branch per stage picks a loop body whose
        // taps are unrolled, so that all fragment reads of a step are in flight before its MFMAs
        auto rows = [&](auto nts_tag) {
            constexpr int NTS = decltype(nts_tag)::value;
            for (int tr = 0; tr < a.TR; ++tr) {
                const int bl = tr >> a.logTI, li = tr & (a.TI - 1);
                if (b0 + bl >= g.B || i0 + li >= g.H) continue;  // uniform
                const float* ap = dys + a_lane + (bl * a.LR + 2 * li) * a.cols;
                const float* bp = xs + b_lane + tr * a.TJ;
                auto step = [&](int sp) {
                    float bv[NC], av[NTS > 0 ? NTS : 1];
#pragma unroll
                    for (int nc = 0; nc < NC; ++nc) bv[nc] = bp[nc * 32 * a.XP + 2 * sp];
#pragma unroll
                    for (int ts = 0; ts < NTS; ++ts) av[ts] = ap[2 * sp + tapoff[ts]];
#pragma unroll
                    for (int ts = 0; ts < NTS; ++ts)
#pragma unroll
                        for (int nc = 0; nc < NC; ++nc)
                            acc[ts][nc] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[ts], bv[nc], acc[ts][nc], 0, 0, 0);
                };
                int sp = 0;
                for (; sp + 2 <= steps; sp += 2) { step(sp); step(sp + 1); }
                if (sp < steps) step(sp);
            }
        };
        if (nts == TS) rows(std::integral_constant<int, TS>{});
        else rows(std::integral_constant<int, TS - 1>{});
    }

    // accumulator register i: output channel 8*(i/4) + 4*kk + (i%4) of the 32, input channel l32
    float* out = part + (size_t)slice * g.Cout * g.Cin * NN;
#pragma unroll
    for (int ts = 0; ts < TS; ++ts) {
        if (ts >= nts) continue;
        const int t = wave + 4 * ts;
#pragma unroll
        for (int nc = 0; nc < NC; ++nc) {
            const int ci = ci0 + nc * 32 + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int co = co0 + 8 * (i / 4) + 4 * kk + (i % 4);
                if (co < g.Cout && ci < g.Cin) out[((size_t)co * NN + t) * g.Cin + ci] = acc[ts][nc][i];
            }
        }
    }
}

// dw[co][ci][tap] = sum over the copies of part[copy][co][tap][ci], copies added in a fixed order;
// threads run along the copies' layout (coalesced reads), the single write pass is scattered
__global__ __launch_bounds__(256) void ukst_sum_taps_kernel(const float* __restrict__ part,
                                                           float* __restrict__ dw, int n, int copies,
                                                           int NN, int Cin)
{
    const int s = blockIdx.x * 256 + threadIdx.x;
    if (s >= n) return;
    // four running sums (copies k, k+1, k+2, k+3 in turn): four loads in flight
    float v4[4] = {0.f, 0.f, 0.f, 0.f};
    int k = 0;
    for (; k + 3 < copies; k += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) v4[u] += part[(size_t)(k + u) * n + s];
    }
    for (int u = 0; k < copies; ++k, ++u) v4[u] += part[(size_t)k * n + s];
    const float v = (v4[0] + v4[1]) + (v4[2] + v4[3]);
    const int ci = s % Cin, r = s / Cin;
    const int tap = r % NN, co = r / NN;
    dw[((size_t)co * Cin + ci) * NN + tap] = v;
}

template <int NC>
bool gw_mfma_args(const Geom& g, GwMfmaArgs& a)
{
    const int N = g.n, CI_T = 32 * NC;
    if (g.Cin < 32 || g.Cout < 32 || N < 2) return false;
    a.g = g;
    a.TJ = pow2_ceil(g.W < 32 ? g.W : 32);
    if (a.TJ < 2) a.TJ = 2;
    a.logTJ = log2_of(a.TJ);
    a.HC = a.TJ + N / 2;
    a.cols = 2 * a.HC;
    const size_t budget = 78 * 1024;
    int TR = 512 / a.TJ;  // at most 512 pixels per stage
    for (;; TR >>= 1) {
        if (TR < 1) return false;
        a.TI = pow2_ceil(g.H < TR ? g.H : TR);
        a.TB = TR / a.TI;
        a.LR = 2 * a.TI + N - 2;
        a.DP = (a.TB * a.LR * a.cols) | 1;
        a.XP = (TR * a.TJ) | 1;
        if ((size_t)4 * (CI_T * a.XP + 32 * a.DP) <= budget) break;
    }
    a.TR = TR;
    a.logTI = log2_of(a.TI);
    a.logPix = log2_of(TR * a.TJ);
    a.tilesX = (g.W + a.TJ - 1) / a.TJ;
    a.tilesY = (g.H + a.TI - 1) / a.TI;
    const long long stages = (long long)a.tilesX * a.tilesY * ((g.B + a.TB - 1) / a.TB);
    if (stages > 0x7fffffffLL) return false;
    a.nStages = (int)stages;
    a.coTiles = (g.Cout + 31) / 32;
    a.ciTiles = (g.Cin + CI_T - 1) / CI_T;
    long long want = 512 / ((long long)a.coTiles * a.ciTiles);
    if (want < 1) want = 1;
    if (want > stages) want = stages;
    a.stagesPerSlice = (int)((stages + want - 1) / want);
    a.nSlices = (int)((stages + a.stagesPerSlice - 1) / a.stagesPerSlice);
    a.cols4 = (a.cols + 3) / 4;
    a.npass = (a.TB * a.LR * a.cols4 + 63) / 64;
    // piecewise staging: rows of at least four elements (a row-end piece is fetched from inside
    // the row), tiles of at least four columns, single buffer descriptors (4 bytes per element
    // bounds both operand types)
    a.fast = (g.W >= 4 && g.OW >= 4 && a.TJ >= 4 && (size_t)g.B * g.Cin * g.H * g.W * 4 <= 0x7FFFFFF0u &&
              (size_t)g.B * g.Cout * g.OH * g.OW * 4 <= 0x7FFFFFF0u) ? 1 : 0;
    a.dC4 = make_fastdiv((unsigned)a.cols4);
    a.dRows = make_fastdiv((unsigned)(a.TB * a.LR));
    a.dLR = make_fastdiv((unsigned)a.LR);
    if ((size_t)g.Cout * g.Cin * N * N > 0x7fffffffu) return false;
    return true;
}

constexpr int gw_nc(int n) { return n <= 4 ? 2 : 1; }  // accumulator tiles per tap by kernel side

template <int N, typename TIn>
hipError_t launch_gw_mfma(const GwMfmaArgs& a, const void* x, const void* dy, float* dw, Workspace& ws,
                          hipStream_t stream)
{
    constexpr int NC = gw_nc(N);
    const GeomBase& g = a.g;
    const size_t elems = (size_t)g.Cout * g.Cin * N * N;
    const size_t need = elems * a.nSlices * sizeof(float);  // one copy of dw per slice
    if (ws.query) { ws.need = need; return hipSuccess; }
    if (ws.bytes < need) return kWorkspaceTooSmall;
    float* part = (float*)ws.ptr;
    hipError_t e;
    const size_t lds = (size_t)4 * (32 * NC * a.XP + 32 * a.DP);
    const void* kfn = (const void*)ukst_grad_weight_mfma_kernel<N, NC, TIn>;
    e = hipFuncSetAttribute(kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) {
        const unsigned nb = (unsigned)((long long)a.nSlices * a.coTiles * a.ciTiles);
        hipLaunchKernelGGL((ukst_grad_weight_mfma_kernel<N, NC, TIn>), dim3(nb), dim3(256), lds, stream,
                           (const TIn*)x, (const TIn*)dy, part, a);
        e = hipGetLastError();
    }
    if (e == hipSuccess) {
        hipLaunchKernelGGL(ukst_sum_taps_kernel, dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, stream,
                           (const float*)part, dw, (int)elems, a.nSlices, N * N, g.Cin);
        e = hipGetLastError();
    }
    return e;
}

// ------------------------------------------------------------------------------------------
// Gradient with respect to the kernel on the bf16 matrix pipe (bf16 layers, 2 <= n <= 4, rows of
// 8-element pieces: W % 8 == 0).
//
// The same product as above, DW_tap[co][ci] += sum_pixel DY_tap[co][pixel] * X[ci][pixel], with the
// pixel axis as the K axis of v_mfma_f32_32x32x16_bf16: a lane's operand is 8 consecutive pixels of
// one channel, which is how NCHW rows lie in memory, so x goes to LDS as it is (16-byte pieces) and
// dy rows are split by column parity on the way (one v_perm pair per piece), which makes the 8
// pixels of any tap consecutive too.  A tap's lattice starts 0 or 1 elements into its half row:
// half of the dy fragments are 16-byte LDS reads at a 2-byte-aligned address (the hardware's
// unaligned DS access; no second, shifted copy of the tile is kept).  Tiles, slices, the dealing
// of taps to waves and the partial-sum layout are those of the fp32 kernel above.
struct GwB16Args {
    GeomBase g;
    int TJ, logTJ, TI, logTI, TB, TR, logPix;  // logPix = log2(TR * TJ)
    int LR, HC, cols, DP, XP;                  // in bf16 elements
    int tilesX, tilesY, nStages, stagesPerSlice, nSlices;
    int coTiles, ciTiles;
    int c8;                                    // 8-column pieces per staged dy row
    int npass;                                 // passes of 64 lanes over a channel's (row, piece) pairs
    FastDiv dC8, dRows, dLR;
};


// 8 packed 16-bit elements moved s places up (s > 0) or down (s < 0), zeros moving in; 0 < |s| < 8
__device__ __forceinline__ gw_u4 shift_elements(gw_u4 v, int s)
{
    unsigned long long lo = v.x | ((unsigned long long)v.y << 32), hi = v.z | ((unsigned long long)v.w << 32);
    if (s > 0) {
        const int sh = 16 * s;
        if (sh >= 64) { hi = lo << (sh - 64); lo = 0; }
        else { hi = (hi << sh) | (lo >> (64 - sh)); lo <<= sh; }
    } else {
        const int sh = -16 * s;
        if (sh >= 64) { lo = hi >> (sh - 64); hi = 0; }
        else { lo = (lo >> sh) | (hi << (64 - sh)); hi >>= sh; }
    }
    return gw_u4{(unsigned)lo, (unsigned)(lo >> 32), (unsigned)hi, (unsigned)(hi >> 32)};
}

template <int N, int NC>
__global__ __launch_bounds__(256, 2) void ukst_grad_weight_mfma_bf16_kernel(const uint16_t* __restrict__ x,
                                                                           const uint16_t* __restrict__ dy,
                                                                           float* __restrict__ part, GwB16Args a)
{
    constexpr int NN = N * N, TS = (NN + 3) / 4, CI_T = 32 * NC;
    extern __shared__ __align__(16) unsigned char lds_b[];
    const GeomBase& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kk = lane >> 5;
    uint16_t* xs = reinterpret_cast<uint16_t*>(lds_b);  // [CI_T][XP]
    uint16_t* dys = xs + CI_T * a.XP;                   // [32][DP]
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
        (void*)x, 0, (int)((size_t)g.B * g.Cin * g.H * g.W * 2), kGwRsrcFlags);
    const __amdgpu_buffer_rsrc_t rs_dy = __builtin_amdgcn_make_buffer_rsrc(
        (void*)dy, 0, (int)((size_t)g.B * g.Cout * g.OH * g.OW * 2), kGwRsrcFlags);

    int bid = xcd_contiguous(blockIdx.x, gridDim.x);  // neighbours in this numbering share an L2
    const int cit = bid % a.ciTiles; bid /= a.ciTiles;
    const int cot = bid % a.coTiles; bid /= a.coTiles;
    const int slice = bid;
    const int co0 = cot * 32, ci0 = cit * CI_T;

    const int nts = (NN - wave + 3) / 4;   // taps of this wave: wave, wave + 4, ...
    int tapoff[TS];
#pragma unroll
    for (int ts = 0; ts < TS; ++ts) {
        const int t = wave + 4 * ts < NN ? wave + 4 * ts : 0;
        const int ta = t / N, tc = t % N;
        tapoff[ts] = (N - 1 - ta) * a.cols + ((N - 1 - tc) & 1) * a.HC + ((N - 1 - tc) >> 1);
    }
    f32x16 acc[TS][NC];
#pragma unroll
    for (int ts = 0; ts < TS; ++ts)
#pragma unroll
        for (int nc = 0; nc < NC; ++nc)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ts][nc][i] = 0.f;

    const int npix = 1 << a.logPix, rowsPerCo = a.TB * a.LR;
    const int a_lane = l32 * a.DP + 8 * kk, b_lane = l32 * a.XP + 8 * kk;
    const int st_end = (slice + 1) * a.stagesPerSlice < a.nStages ? (slice + 1) * a.stagesPerSlice : a.nStages;
    for (int st = slice * a.stagesPerSlice; st < st_end; ++st) {
        int t = st;
        const int tx = t % a.tilesX; t /= a.tilesX;
        const int ty = t % a.tilesY; t /= a.tilesY;
        const int b0 = t * a.TB, i0 = ty * a.TI, j0 = tx * a.TJ;
        const int oy_base = 2 * i0 + g.P - (N - 1), ox_base = 2 * j0 + g.P - (N - 1);
        __syncthreads();
        // Staging without divergent address arithmetic per piece: every wave owns a quarter of
        // the channels; what depends on the lane (row, piece, validity) is worked out once per
        // stage, the channel enters through the scalar offset of a buffer load, and all loads of
        // a group are in flight before the first LDS write.  Rows, images and channels that do
        // not exist are read through an out-of-range offset and arrive as zeros.
        // dy tile: 8 columns per piece, split by column parity: column cc of a row sits at
        // (cc & 1) * HC + (cc >> 1).  A piece that hangs over the left or right end of its row is
        // fetched from inside the row and shifted into place (zeros move in).  Per pass of 64
        // lanes over a channel's (row, piece) pairs: the lane's part of the address, then the
        // wave's 8 channels in two groups; a group's loads are requested before the previous
        // group is written, so one memory round trip covers the whole stage.
        constexpr int GRP = 4;
        const int per_co = rowsPerCo * a.c8;
        const unsigned co_bytes = (unsigned)(g.OH * g.OW * 2);
        unsigned dvoff;
        int dsh, ddst;
        auto lane_pass = [&](int pp) {
            const int idx = lane + 64 * pp;
            const int rem = fdiv(idx, a.dC8), m = idx - rem * a.c8;
            const int bl = fdiv(rem, a.dLR), rr = rem - bl * a.LR;
            const int b = b0 + bl, oy = oy_base + rr, ox = ox_base + 8 * m;
            const bool ok = idx < per_co && b < g.B && oy >= 0 && oy < g.OH && ox + 7 >= 0 && ox < g.OW;
            const int oxl = ox < 0 ? 0 : (ox > g.OW - 8 ? g.OW - 8 : ox);
            dsh = oxl - ox;
            dvoff = ok ? (unsigned)((((b * g.Cout) * g.OH + oy) * g.OW + oxl) * 2) : kGwInvalid;
            ddst = idx < per_co ? rem * a.cols + 4 * m : -1;
        };
        auto load_group = [&](int h, gw_u4 (&q)[GRP]) {
#pragma unroll
            for (int c4 = 0; c4 < GRP; ++c4) {
                const int co = co0 + wave * 8 + h * GRP + c4;  // uniform
                const bool cok = co < g.Cout;
                q[c4] = __builtin_amdgcn_raw_buffer_load_b128(rs_dy, cok ? dvoff : kGwInvalid,
                                                              cok ? (unsigned)co * co_bytes : 0u, 0);
            }
        };
        auto write_group = [&](int h, int sh, int dst, const gw_u4 (&q)[GRP]) {
            if (dst < 0) return;
#pragma unroll
            for (int c4 = 0; c4 < GRP; ++c4) {
                uint16_t* base = dys + (wave * 8 + h * GRP + c4) * a.DP + dst;
                gw_u4 v = q[c4];
                if (sh != 0) v = shift_elements(v, sh);
                const gw_u2 ev = {__builtin_amdgcn_perm(v.y, v.x, 0x05040100u),
                                  __builtin_amdgcn_perm(v.w, v.z, 0x05040100u)};
                const gw_u2 od = {__builtin_amdgcn_perm(v.y, v.x, 0x07060302u),
                                  __builtin_amdgcn_perm(v.w, v.z, 0x07060302u)};
                *reinterpret_cast<gw_u2*>(base) = ev;
                *reinterpret_cast<gw_u2*>(base + a.HC) = od;
            }
        };
        gw_u4 qa[GRP], qb[GRP];
        lane_pass(0);
        load_group(0, qa);
        {
            // x tile: 8 pixels of a row per piece; W % 8 == 0, so a piece lies in the row or past it
            const int logCPC = a.logPix - 3, CPC = 1 << logCPC;  // pieces per channel
            const int cw0 = wave * (CI_T / 4);
            const int xpasses = ((CI_T / 4) << logCPC) >> 6;     // >= 2
            for (int p0 = 0; p0 < xpasses; p0 += 4) {
                gw_u4 q[4];
                int dst[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    dst[u] = -1;
                    if (p0 + u < xpasses) {
                        const int flat = lane + 64 * (p0 + u);
                        const int cl = cw0 + (flat >> logCPC), pix = (flat & (CPC - 1)) << 3;
                        const int tr = pix >> a.logTJ, lj = pix & (a.TJ - 1);
                        const int b = b0 + (tr >> a.logTI), i = i0 + (tr & (a.TI - 1)), j = j0 + lj, ci = ci0 + cl;
                        const bool ok = ci < g.Cin && b < g.B && i < g.H && j < g.W;
                        const unsigned voff = ok ? (unsigned)((((b * g.Cin + ci) * g.H + i) * g.W + j) * 2) : kGwInvalid;
                        q[u] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, voff, 0, 0);
                        dst[u] = cl * a.XP + pix;
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (dst[u] >= 0) *reinterpret_cast<gw_u4*>(xs + dst[u]) = q[u];
            }
        }
#pragma unroll 1
        for (int pp = 0; pp < a.npass; ++pp) {
            const int sh_c = dsh, dst_c = ddst;
            load_group(1, qb);
            write_group(0, sh_c, dst_c, qa);
            if (pp + 1 < a.npass) {
                lane_pass(pp + 1);
                load_group(0, qa);
            }
            write_group(1, sh_c, dst_c, qb);
        }
        __syncthreads();
        // K steps of 16 pixels along a row; pixels past the end of the row are zeros in x
        const int wj = g.W - j0 < a.TJ ? g.W - j0 : a.TJ;
        const int steps = (wj + 15) >> 4;
        // the tap count of a wave is TS or TS - 1: one branch per stage picks a loop body whose
        // taps are unrolled, so that all fragment reads of a step are in flight before its MFMAs
        auto rows = [&](auto nts_tag) {
            constexpr int NTS = decltype(nts_tag)::value;
            for (int tr = 0; tr < a.TR; ++tr) {
                const int bl = tr >> a.logTI, li = tr & (a.TI - 1);
                if (b0 + bl >= g.B || i0 + li >= g.H) continue;  // uniform
                const uint16_t* ap = dys + a_lane + (bl * a.LR + 2 * li) * a.cols;
                const uint16_t* bp = xs + b_lane + tr * a.TJ;
                for (int sp = 0; sp < steps; ++sp) {
                    gw_bf16x8 bv[NC], av[NTS > 0 ? NTS : 1];
#pragma unroll
                    for (int nc = 0; nc < NC; ++nc)
                        bv[nc] = *reinterpret_cast<const gw_bf16x8*>(bp + nc * 32 * a.XP + 16 * sp);
#pragma unroll
                    for (int ts = 0; ts < NTS; ++ts)
                        av[ts] = *reinterpret_cast<const gw_bf16x8u*>(ap + 16 * sp + tapoff[ts]);
#pragma unroll
                    for (int ts = 0; ts < NTS; ++ts)
#pragma unroll
                        for (int nc = 0; nc < NC; ++nc)
                            acc[ts][nc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[ts], bv[nc], acc[ts][nc], 0, 0, 0);
                }
            }
        };
        if (nts == TS) rows(std::integral_constant<int, TS>{});
        else rows(std::integral_constant<int, TS - 1>{});
    }

    // accumulator register i: output channel 8*(i/4) + 4*kk + (i%4) of the 32, input channel l32
    float* out = part + (size_t)slice * g.Cout * g.Cin * NN;
#pragma unroll
    for (int ts = 0; ts < TS; ++ts) {
        if (ts >= nts) continue;
        const int t = wave + 4 * ts;
#pragma unroll
        for (int nc = 0; nc < NC; ++nc) {
            const int ci = ci0 + nc * 32 + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int co = co0 + 8 * (i / 4) + 4 * kk + (i % 4);
                if (co < g.Cout && ci < g.Cin) out[((size_t)co * NN + t) * g.Cin + ci] = acc[ts][nc][i];
            }
        }
    }
}

constexpr int GW_B16_NC = 2;

bool gw_b16_args(const Geom& g, GwB16Args& a)
{
    const int N = g.n, CI_T = 32 * GW_B16_NC;
    if (g.Cin < 32 || g.Cout < 32 || N < 2 || N > 4) return false;
    if (g.W % 8 != 0 || g.W < 16) return false;
    a.g = g;
    a.TJ = g.W >= 32 ? 32 : 16;
    a.logTJ = log2_of(a.TJ);
    a.HC = a.TJ + 8;  // half rows: TJ + 1 columns are read, TJ + 4 written, 16-byte multiples
    a.cols = 2 * a.HC;
    a.c8 = (2 * a.TJ + N - 2 + 7) / 8;
    const size_t budget = 78 * 1024;
    int TR = 512 / a.TJ;  // at most 512 pixels per stage
    for (;; TR >>= 1) {
        if (TR < 1) return false;
        a.TI = pow2_ceil(g.H < TR ? g.H : TR);
        a.TB = TR / a.TI;
        a.LR = 2 * a.TI + N - 2;
        // channel strides: a multiple of 8 elements (16-byte pieces) whose count of pieces is odd,
        // so that the 16 lanes of a read pass fall into different bank groups
        a.DP = a.TB * a.LR * a.cols;
        if ((a.DP / 8) % 2 == 0) a.DP += 8;
        a.XP = TR * a.TJ + 8;
        if ((size_t)2 * (CI_T * a.XP + 32 * a.DP) <= budget) break;
    }
    a.TR = TR;
    a.logTI = log2_of(a.TI);
    a.logPix = log2_of(TR * a.TJ);
    a.tilesX = (g.W + a.TJ - 1) / a.TJ;
    a.tilesY = (g.H + a.TI - 1) / a.TI;
    const long long stages = (long long)a.tilesX * a.tilesY * ((g.B + a.TB - 1) / a.TB);
    if (stages > 0x7fffffffLL) return false;
    a.nStages = (int)stages;
    a.coTiles = (g.Cout + 31) / 32;
    a.ciTiles = (g.Cin + CI_T - 1) / CI_T;
    long long want = 512 / ((long long)a.coTiles * a.ciTiles);
    if (want < 1) want = 1;
    if (want > stages) want = stages;
    a.stagesPerSlice = (int)((stages + want - 1) / want);
    a.nSlices = (int)((stages + a.stagesPerSlice - 1) / a.stagesPerSlice);
    a.dC8 = make_fastdiv((unsigned)a.c8);
    a.dRows = make_fastdiv((unsigned)(a.TB * a.LR));
    a.dLR = make_fastdiv((unsigned)a.LR);
    if ((size_t)g.Cout * g.Cin * N * N > 0x7fffffffu) return false;
    a.npass = (a.TB * a.LR * a.c8 + 63) / 64;
    if (g.OW < 8) return false;
    // single buffer descriptors, 32-bit byte offsets
    if ((size_t)g.B * g.Cin * g.H * g.W * 2 > 0x7FFFFFF0u || (size_t)g.B * g.Cout * g.OH * g.OW * 2 > 0x7FFFFFF0u)
        return false;
    return true;
}

template <int N>
hipError_t launch_gw_b16(const GwB16Args& a, const void* x, const void* dy, float* dw, Workspace& ws,
                         hipStream_t stream)
{
    constexpr int NC = GW_B16_NC;
    const GeomBase& g = a.g;
    const size_t elems = (size_t)g.Cout * g.Cin * N * N;
    const size_t need = elems * a.nSlices * sizeof(float);  // one copy of dw per slice
    if (ws.query) { ws.need = need; return hipSuccess; }
    if (ws.bytes < need) return kWorkspaceTooSmall;
    float* part = (float*)ws.ptr;
    hipError_t e;
    const size_t lds = (size_t)2 * (32 * NC * a.XP + 32 * a.DP);
    const void* kfn = (const void*)ukst_grad_weight_mfma_bf16_kernel<N, NC>;
    e = hipFuncSetAttribute(kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) {
        const unsigned nb = (unsigned)((long long)a.nSlices * a.coTiles * a.ciTiles);
        hipLaunchKernelGGL((ukst_grad_weight_mfma_bf16_kernel<N, NC>), dim3(nb), dim3(256), lds, stream,
                           (const uint16_t*)x, (const uint16_t*)dy, part, a);
        e = hipGetLastError();
    }
    if (e == hipSuccess) {
        hipLaunchKernelGGL(ukst_sum_taps_kernel, dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, stream,
                           (const float*)part, dw, (int)elems, a.nSlices, N * N, g.Cin);
        e = hipGetLastError();
    }
    return e;
}

// ------------------------------------------------------------------------------------------
// Gradient with respect to the kernel for layers with few output channels, on the matrix cores
// (Cout * n*n <= 64: the last layer of a generator, 64 -> 3 channels; image-to-image layers).
//
// With so few output channels the channel axis cannot fill an MFMA tile, but (channel, tap) pairs
// can -- the mirror image of the thin forward kernel: row r = co * n*n + tap of
//     DW[r][ci] += sum_pixel DY_r[pixel] * X[ci][pixel],     DY_r[pixel] = dy[co][2i+P-a][2j+P-c]
// is one row of a v_mfma_f32_32x32x2_f32 tile, each lane reading its own shifted view of the
// parity-split dy tile.  The four waves of a block take every fourth pixel row of a stage, keep
// MT x CT accumulator tiles each, and add them through LDS in wave order at the end of the block's
// slice; blocks write one copy of dw per slice (dw's own layout), ukst_sum_partials_kernel adds
// the copies in a fixed order.  Staging is the piecewise one of the kernels above.
struct GwThinArgs {
    GeomBase g;
    int TJ, logTJ, TI, logTI, TB, TR, logPix;  // logPix = log2(TR * TJ)
    int LR, HC, cols, DP, XP;
    int tilesX, tilesY, nStages, stagesPerSlice, nSlices;
    int ciTiles;
    int cols4, npass;
    FastDiv dC4, dLR;
};

template <int N, int MT, int CT, typename TIn>
__global__ __launch_bounds__(256, 2) void ukst_grad_weight_thin_mfma_kernel(const TIn* __restrict__ x,
                                                                           const TIn* __restrict__ dy,
                                                                           float* __restrict__ part, GwThinArgs a)
{
    constexpr int NN = N * N, CI_T = 32 * CT;
    constexpr int ES = (int)sizeof(TIn);
    extern __shared__ __align__(16) float lds_f[];
    const GeomBase& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kk = lane >> 5;
    float* xs = lds_f;                     // [CI_T][XP]
    float* dys = lds_f + CI_T * a.XP;      // [Cout][DP]
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
        (void*)x, 0, (int)((size_t)g.B * g.Cin * g.H * g.W * ES), kGwRsrcFlags);
    const __amdgpu_buffer_rsrc_t rs_dy = __builtin_amdgcn_make_buffer_rsrc(
        (void*)dy, 0, (int)((size_t)g.B * g.Cout * g.OH * g.OW * ES), kGwRsrcFlags);

    int bid = xcd_contiguous(blockIdx.x, gridDim.x);
    const int cit = bid % a.ciTiles; bid /= a.ciTiles;
    const int slice = bid;
    const int ci0 = cit * CI_T;

    // this lane's rows (channel, tap): LDS offset of its view of the dy tile, -1 if the row does not exist
    int arow[MT];
#pragma unroll
    for (int mi = 0; mi < MT; ++mi) {
        const int r = mi * 32 + l32, co = r / NN, t = r - co * NN;
        const int ta = t / N, tc = t - ta * N;
        arow[mi] = co < g.Cout ? co * a.DP + (N - 1 - ta) * a.cols + ((N - 1 - tc) & 1) * a.HC + ((N - 1 - tc) >> 1) + kk
                               : -1;
    }
    f32x16 acc[MT][CT];
#pragma unroll
    for (int mi = 0; mi < MT; ++mi)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ct][i] = 0.f;

    const int rowsPerCo = a.TB * a.LR;
    const int b_lane = l32 * a.XP + kk;
    auto load_piece = [&](const __amdgpu_buffer_rsrc_t& rs, unsigned voff, unsigned soff) -> Quad {
        if constexpr (ES == 4) {
            const gw_u4 t = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soff, 0);
            return Quad{{__uint_as_float(t.x), __uint_as_float(t.y), __uint_as_float(t.z), __uint_as_float(t.w)}};
        } else {
            const gw_u2 t = __builtin_amdgcn_raw_buffer_load_b64(rs, voff, soff, 0);
            return Quad{{__uint_as_float(t.x << 16), __uint_as_float(t.x & 0xFFFF0000u),
                         __uint_as_float(t.y << 16), __uint_as_float(t.y & 0xFFFF0000u)}};
        }
    };
    // four elements moved sh places up (sh > 0) or down, zeros moving in; 0 < |sh| < 4
    auto shifted = [&](const Quad& q, int sh) -> Quad {
        Quad r;
#pragma unroll
        for (int k2 = 0; k2 < 4; ++k2) {
            const int src = k2 - sh;
            float v = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) v = src == e ? q.v[e] : v;
            r.v[k2] = v;
        }
        return r;
    };
    const int st_end = (slice + 1) * a.stagesPerSlice < a.nStages ? (slice + 1) * a.stagesPerSlice : a.nStages;
    for (int st = slice * a.stagesPerSlice; st < st_end; ++st) {
        int t = st;
        const int tx = t % a.tilesX; t /= a.tilesX;
        const int ty = t % a.tilesY; t /= a.tilesY;
        const int b0 = t * a.TB, i0 = ty * a.TI, j0 = tx * a.TJ;
        const int oy_base = 2 * i0 + g.P - (N - 1), ox_base = 2 * j0 + g.P - (N - 1);
        __syncthreads();
        // All loads of a batch (four x pieces per lane, with the first batch four dy pieces) are
        // requested before the first LDS write.
        const int logCPC = a.logPix - 2, CPC = 1 << logCPC;  // x pieces per channel
        const int cw0 = wave * (CI_T / 4);
        const int xpasses = (((CI_T / 4) << logCPC) + 63) >> 6;
        const int per_co = rowsPerCo * a.cols4;
        const unsigned dsoff = (unsigned)wave * (unsigned)(g.OH * g.OW * ES);
        float* dbase = dys + wave * a.DP;
        auto x_load = [&](int pass, Quad& q, int& dst, int& sh) {
            dst = -1;
            sh = 0;
            const int flat = lane + 64 * pass;
            if (pass < xpasses && (flat >> logCPC) < CI_T / 4) {
                const int cl = cw0 + (flat >> logCPC), pix = (flat & (CPC - 1)) << 2;
                const int tr = pix >> a.logTJ, lj = pix & (a.TJ - 1);
                const int b = b0 + (tr >> a.logTI), i = i0 + (tr & (a.TI - 1)), j = j0 + lj, ci = ci0 + cl;
                const bool ok = ci < g.Cin && b < g.B && i < g.H && j < g.W;
                const int jl = j > g.W - 4 ? g.W - 4 : j;
                sh = jl - j;
                const unsigned voff = ok ? (unsigned)((((b * g.Cin + ci) * g.H + i) * g.W + jl) * ES) : kGwInvalid;
                q = load_piece(rs_x, voff, 0u);
                dst = cl * a.XP + pix;
            }
        };
        auto x_store = [&](const Quad& q, int dst, int sh) {
            if (dst < 0) return;
            const Quad v = sh != 0 ? shifted(q, sh) : q;
#pragma unroll
            for (int k2 = 0; k2 < 4; ++k2) xs[dst + k2] = v.v[k2];
        };
        // dy tile: wave w stages output channel w (there are at most four)
        auto d_load = [&](int pass, Quad& q, int& dst, int& sh, int& nc) {
            const int idx = lane + 64 * pass;
            dst = -1;
            sh = 0;
            nc = 0;
            if (wave < g.Cout && idx < per_co) {
                const int rem = fdiv(idx, a.dC4), m = idx - rem * a.cols4;
                const int bl = fdiv(rem, a.dLR), rr = rem - bl * a.LR;
                const int b = b0 + bl, oy = oy_base + rr, ox = ox_base + 4 * m;
                const bool ok = b < g.B && oy >= 0 && oy < g.OH && ox + 3 >= 0 && ox < g.OW;
                const int oxl = ox < 0 ? 0 : (ox > g.OW - 4 ? g.OW - 4 : ox);
                sh = oxl - ox;
                const unsigned voff = ok ? (unsigned)((((b * g.Cout) * g.OH + oy) * g.OW + oxl) * ES) : kGwInvalid;
                q = load_piece(rs_dy, voff, dsoff);
                dst = rem * a.cols + 2 * m;
                nc = a.cols - 4 * m;
            }
        };
        auto d_store = [&](const Quad& q, int dst, int sh, int nc) {
            if (dst < 0) return;
            const Quad v = sh != 0 ? shifted(q, sh) : q;
            dbase[dst] = v.v[0];
            dbase[dst + a.HC] = v.v[1];
            if (nc > 2) {
                dbase[dst + 1] = v.v[2];
                dbase[dst + a.HC + 1] = v.v[3];
            }
        };
        {
            Quad xq[4], dq[4];
            int xd[4], xsft[4], dd[4], dsft[4], dn[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) x_load(u, xq[u], xd[u], xsft[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) d_load(u, dq[u], dd[u], dsft[u], dn[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) x_store(xq[u], xd[u], xsft[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) d_store(dq[u], dd[u], dsft[u], dn[u]);
        }
        for (int p0 = 4; p0 < xpasses; p0 += 4) {  // further batches
            Quad xq[4];
            int xd[4], xsft[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) x_load(p0 + u, xq[u], xd[u], xsft[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) x_store(xq[u], xd[u], xsft[u]);
        }
        for (int p0 = 4; p0 < a.npass; p0 += 4) {
            Quad dq[4];
            int dd[4], dsft[4], dn[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) d_load(p0 + u, dq[u], dd[u], dsft[u], dn[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) d_store(dq[u], dd[u], dsft[u], dn[u]);
        }
        __syncthreads();
        const int wj = g.W - j0 < a.TJ ? g.W - j0 : a.TJ;
        const int steps = (wj + 1) >> 1;
        for (int tr = wave; tr < a.TR; tr += 4) {  // every fourth pixel row of the stage
            const int bl = tr >> a.logTI, li = tr & (a.TI - 1);
            if (b0 + bl >= g.B || i0 + li >= g.H) continue;  // uniform
            const float* ap = dys + (bl * a.LR + 2 * li) * a.cols;
            const float* bp = xs + b_lane + tr * a.TJ;
            for (int sp = 0; sp < steps; ++sp) {
                float bv[CT], av[MT];
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) bv[ct] = bp[ct * 32 * a.XP + 2 * sp];
#pragma unroll
                for (int mi = 0; mi < MT; ++mi) av[mi] = arow[mi] >= 0 ? ap[arow[mi] + 2 * sp] : 0.f;
#pragma unroll
                for (int mi = 0; mi < MT; ++mi)
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct)
                        acc[mi][ct] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[mi], bv[ct], acc[mi][ct], 0, 0, 0);
            }
        }
    }

    // the four waves' sums meet in LDS: waves 1..3 park theirs, wave 0 adds them in that order
    __syncthreads();
    constexpr int TILE = 16 * 64;  // floats of one accumulator tile over the wave
    if (wave > 0) {
#pragma unroll
        for (int mi = 0; mi < MT; ++mi)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    lds_f[((wave - 1) * MT * CT + mi * CT + ct) * TILE + i * 64 + lane] = acc[mi][ct][i];
    }
    __syncthreads();
    if (wave != 0) return;
    // accumulator register i: row 8*(i/4) + 4*kk + (i%4) of the tile's 32, input channel l32
    float* out = part + (size_t)slice * g.Cout * g.Cin * NN;
#pragma unroll
    for (int mi = 0; mi < MT; ++mi)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            const int ci = ci0 + ct * 32 + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float v = acc[mi][ct][i];
#pragma unroll
                for (int w2 = 0; w2 < 3; ++w2) v += lds_f[(w2 * MT * CT + mi * CT + ct) * TILE + i * 64 + lane];
                const int r = mi * 32 + 8 * (i / 4) + 4 * kk + (i % 4);
                const int co = r / NN, tap = r - co * NN;
                if (co < g.Cout && ci < g.Cin) out[((size_t)co * g.Cin + ci) * NN + tap] = v;
            }
        }
}

template <int N>
bool gw_thin_args(const Geom& g, GwThinArgs& a, int CT)
{
    constexpr int NN = N * N;
    if (g.Cout > 4 || g.Cout * NN > 64) return false;
    if (g.Cin < 16) return false;  // fewer input channels leave the MFMA columns empty: the vector ALUs are faster
    if (g.W < 4 || g.OW < 4) return false;  // piecewise staging: rows of at least four elements
    if ((size_t)g.B * g.Cin * g.H * g.W * 4 > 0x7FFFFFF0u || (size_t)g.B * g.Cout * g.OH * g.OW * 4 > 0x7FFFFFF0u)
        return false;
    const int CI_T = 32 * CT;
    a.g = g;
    a.TJ = pow2_ceil(g.W < 32 ? g.W : 32);
    if (a.TJ < 4) a.TJ = 4;
    a.logTJ = log2_of(a.TJ);
    a.HC = a.TJ + N / 2;
    a.cols = 2 * a.HC;
    const size_t budget = 64 * 1024;
    int TR = 256 / a.TJ;  // at most 256 pixels per stage; at least 4 rows so that every wave has one
    if (TR < 4) TR = 4;
    for (;; TR >>= 1) {
        if (TR < 4) return false;
        a.TI = pow2_ceil(g.H < TR ? g.H : TR);
        a.TB = TR / a.TI;
        a.LR = 2 * a.TI + N - 2;
        a.DP = (a.TB * a.LR * a.cols) | 1;
        a.XP = (TR * a.TJ) | 1;
        if ((size_t)4 * (CI_T * a.XP + g.Cout * a.DP) <= budget) break;
    }
    a.TR = TR;
    a.logTI = log2_of(a.TI);
    a.logPix = log2_of(TR * a.TJ);
    a.tilesX = (g.W + a.TJ - 1) / a.TJ;
    a.tilesY = (g.H + a.TI - 1) / a.TI;
    const long long stages = (long long)a.tilesX * a.tilesY * ((g.B + a.TB - 1) / a.TB);
    if (stages > 0x7fffffffLL) return false;
    a.nStages = (int)stages;
    a.ciTiles = (g.Cin + CI_T - 1) / CI_T;
    long long want = 1024 / (long long)a.ciTiles;  // blocks to cover the chip four times
    if (want < 1) want = 1;
    if (want > stages) want = stages;
    a.stagesPerSlice = (int)((stages + want - 1) / want);
    a.nSlices = (int)((stages + a.stagesPerSlice - 1) / a.stagesPerSlice);
    a.cols4 = (a.cols + 3) / 4;
    a.npass = (a.TB * a.LR * a.cols4 + 63) / 64;
    a.dC4 = make_fastdiv((unsigned)a.cols4);
    a.dLR = make_fastdiv((unsigned)a.LR);
    if ((size_t)g.Cout * g.Cin * NN > 0x7fffffffu) return false;
    return true;
}

template <int N, int MT, int CT, typename TIn>
hipError_t launch_gw_thin_t(const GwThinArgs& a, const void* x, const void* dy, float* dw, Workspace& ws,
                            hipStream_t stream)
{
    const GeomBase& g = a.g;
    const size_t elems = (size_t)g.Cout * g.Cin * N * N;
    const int copies = a.nSlices;
    const size_t need = elems * copies * sizeof(float);  // one copy of dw per slice
    if (ws.query) { ws.need = need; return hipSuccess; }
    if (ws.bytes < need) return kWorkspaceTooSmall;
    float* part = (float*)ws.ptr;
    size_t lds = (size_t)4 * (32 * CT * a.XP + g.Cout * a.DP);
    const size_t red = (size_t)3 * MT * CT * 16 * 64 * 4;  // three waves' accumulators
    if (lds < red) lds = red;
    const void* kfn = (const void*)ukst_grad_weight_thin_mfma_kernel<N, MT, CT, TIn>;
    hipError_t e = hipFuncSetAttribute(kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const unsigned nb = (unsigned)((long long)a.nSlices * a.ciTiles);
    hipLaunchKernelGGL((ukst_grad_weight_thin_mfma_kernel<N, MT, CT, TIn>), dim3(nb), dim3(256), lds, stream,
                       (const TIn*)x, (const TIn*)dy, part, a);
    e = hipGetLastError();
    if (e == hipSuccess) {
        int logR = 0;  // lanes per element: until the sum kernel has about 64k threads
        while (logR < 8 && (elems << logR) < 65536 && (2 << logR) <= copies) ++logR;
        const unsigned per_block = 256u >> logR;
        hipLaunchKernelGGL(ukst_sum_partials_kernel, dim3((unsigned)((elems + per_block - 1) / per_block)),
                           dim3(256), 0, stream, (const float*)part, dw, (int)elems, copies, logR);
        e = hipGetLastError();
    }
    return e;
}

// true (and a filled description) if the thin matrix-core kernel gradient takes the layer
template <int N>
bool gw_thin_pick(const Geom& g, GwThinArgs& a, int& MT, int& CT)
{
    if constexpr (N < 2 || N > 5) return false;
    else {
        CT = g.Cin > 32 ? 2 : 1;
        MT = g.Cout * N * N > 32 ? 2 : 1;
        return gw_thin_args<N>(g, a, CT);
    }
}

template <int N, typename TIn>
hipError_t launch_gw_thin(const GwThinArgs& a, int MT, int CT, const void* x, const void* dy, float* dw,
                          Workspace& ws, hipStream_t stream)
{
    if (MT == 1 && CT == 1) return launch_gw_thin_t<N, 1, 1, TIn>(a, x, dy, dw, ws, stream);
    if (MT == 1 && CT == 2) return launch_gw_thin_t<N, 1, 2, TIn>(a, x, dy, dw, ws, stream);
    if (MT == 2 && CT == 1) return launch_gw_thin_t<N, 2, 1, TIn>(a, x, dy, dw, ws, stream);
    return launch_gw_thin_t<N, 2, 2, TIn>(a, x, dy, dw, ws, stream);
}

template <int N, int CO_R, int CI_R, typename TIn>
hipError_t launch_gw(const Geom& g, const void* x, const void* dy, float* dw, Workspace& ws,
                     hipStream_t stream)
{
    GradWArgs a;
    a.g = g;
    // channel threads: as many as the layer has pairs for, the rest of the block goes to pixels
    a.TCI = pow2_ceil((g.Cin + CI_R - 1) / CI_R);
    if (a.TCI > 16) a.TCI = 16;
    a.TCO = pow2_ceil((g.Cout + CO_R - 1) / CO_R);
    if (a.TCO > 16) a.TCO = 16;
    a.PB = a.TCO * a.TCI;
    a.TP = 256 / a.PB;
    a.logTCI = log2_of(a.TCI);
    a.logPB = log2_of(a.PB);
    a.SUB = a.PB <= 64 ? 4 : a.PB == 128 ? 2 : 1;
    a.foldWaves = (a.PB <= 64 && 4 * a.PB * CO_R * CI_R * N * N * 4 <= 16 * 1024) ? 1 : 0;
    if (a.foldWaves) a.SUB = 1;
    const int CO_T = a.TCO * CO_R, CI_T = a.TCI * CI_R;
    a.TJ = pow2_ceil(g.W < 32 ? g.W : 32);
    a.logTJ = log2_of(a.TJ);
    // pixel rows per stage: enough pixels for every pixel thread, within the LDS budget
    a.XS = CI_T + (CI_T >= 32 ? 4 : 0);
    a.LC = 2 * a.TJ + N - 2 > 1 ? 2 * a.TJ + N - 2 : 1;
    const size_t budget = 64 * 1024;
    int TI = pow2_ceil(g.H < 64 ? g.H : 64);
    while (TI > 1 && (size_t)4 * (TI * a.TJ * a.XS + CO_T * (2 * TI + N - 2) * a.LC) > budget) TI >>= 1;
    a.TI = TI;
    a.LR = 2 * TI + N - 2 > 1 ? 2 * TI + N - 2 : 1;
    a.LC4 = (a.LC + 3) / 4;
    a.dLC4 = make_fastdiv((unsigned)a.LC4);
    a.dLR = make_fastdiv((unsigned)a.LR);
    size_t lds = (size_t)4 * (TI * a.TJ * a.XS + CO_T * a.LR * a.LC);
    if (lds > budget) return hipErrorInvalidConfiguration;
    if (a.foldWaves && lds < 16 * 1024) lds = 16 * 1024;  // room for the four waves' sums
    a.tilesX = (g.W + a.TJ - 1) / a.TJ;
    a.tilesY = (g.H + TI - 1) / TI;
    const long long stages = (long long)a.tilesX * a.tilesY * g.B;
    if (stages > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    a.nStages = (int)stages;
    a.coTiles = (g.Cout + CO_T - 1) / CO_T;
    a.ciTiles = (g.Cin + CI_T - 1) / CI_T;
    // slices: enough blocks to cover the chip four times (twice when most of a block's threads
    // share channel pairs: each block then ends with a shuffle reduction that wants amortising),
    // never more than stages
    long long want = (a.PB >= 64 ? 1024 : 1024) / ((long long)a.coTiles * a.ciTiles);
    if (want < 1) want = 1;
    if (want > stages) want = stages;
    a.stagesPerSlice = (int)((stages + want - 1) / want);
    a.nSlices = (int)((stages + a.stagesPerSlice - 1) / a.stagesPerSlice);
    const long long nb = (long long)a.nSlices * a.coTiles * a.ciTiles;
    if (nb > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const int copies = a.nSlices * a.SUB;
    const size_t elems = (size_t)g.Cout * g.Cin * N * N;
    if (elems > 0x7fffffffu) return hipErrorInvalidConfiguration;
    const size_t need = elems * copies * sizeof(float);  // one copy of dw per (slice, wave group)
    if (ws.query) { ws.need = need; return hipSuccess; }
    if (ws.bytes < need) return kWorkspaceTooSmall;
    float* part = (float*)ws.ptr;
    hipError_t e;
    hipLaunchKernelGGL((ukst_grad_weight_kernel<N, CO_R, CI_R, TIn>), dim3((unsigned)nb), dim3(256), lds,
                       stream, (const TIn*)x, (const TIn*)dy, part, a);
    e = hipGetLastError();
    if (e == hipSuccess) {
        int logR = 0;  // lanes per element: until the sum kernel has about 64k threads
        while (logR < 8 && (elems << logR) < 65536 && (2 << logR) <= copies) ++logR;
        const unsigned per_block = 256u >> logR;
        hipLaunchKernelGGL(ukst_sum_partials_kernel, dim3((unsigned)((elems + per_block - 1) / per_block)),
                           dim3(256), 0, stream, (const float*)part, dw, (int)elems, copies, logR);
        e = hipGetLastError();
    }
    return e;
}

// register block: CO_R x CI_R channel pairs x n*n taps per thread; layers with at most four
// channels on a side take one channel per thread there, which leaves the block's threads to the
// pixels and keeps the closing shuffle reduction short
template <int N, typename TIn>
hipError_t launch_gw_n(const Geom& g, const void* x, const void* dy, float* dw, Workspace& ws,
                       hipStream_t stream)
{
    if constexpr (N >= 2 && N <= 4 && sizeof(TIn) == 2) {
        GwB16Args ba;  // bf16 layers: the bf16 matrix pipe where the kernel takes the shape
        if (gw_b16_args(g, ba)) return launch_gw_b16<N>(ba, x, dy, dw, ws, stream);
    }
    if constexpr (N >= 2) {
        GwMfmaArgs ma;
        if (gw_mfma_args<gw_nc(N)>(g, ma)) return launch_gw_mfma<N, TIn>(ma, x, dy, dw, ws, stream);
    }
    if constexpr (N >= 2 && N <= 5) {
        GwThinArgs ta;  // few output channels: (channel, tap) pairs as MFMA rows
        int MT = 1, CT = 1;
        if (gw_thin_pick<N>(g, ta, MT, CT)) return launch_gw_thin<N, TIn>(ta, MT, CT, x, dy, dw, ws, stream);
    }
    constexpr int CO_W = N <= 3 ? 4 : N <= 5 ? 2 : 1;  // wide register block: CO_W x 4 pairs
    const bool thin_o = g.Cout <= 4, thin_i = g.Cin <= 4;
    if (thin_o && thin_i) return launch_gw<N, 1, 1, TIn>(g, x, dy, dw, ws, stream);
    if (thin_o) return launch_gw<N, 1, 4, TIn>(g, x, dy, dw, ws, stream);
    if (thin_i) return launch_gw<N, CO_W, 1, TIn>(g, x, dy, dw, ws, stream);
    return launch_gw<N, CO_W, 4, TIn>(g, x, dy, dw, ws, stream);
}

template <typename TIn>
hipError_t launch_gw_t(const Geom& g, const void* x, const void* dy, float* dw, Workspace& ws,
                       hipStream_t stream)
{
    switch (g.n) {
        case 1: return launch_gw_n<1, TIn>(g, x, dy, dw, ws, stream);
        case 2: return launch_gw_n<2, TIn>(g, x, dy, dw, ws, stream);
        case 3: return launch_gw_n<3, TIn>(g, x, dy, dw, ws, stream);
        case 4: return launch_gw_n<4, TIn>(g, x, dy, dw, ws, stream);
        case 5: return launch_gw_n<5, TIn>(g, x, dy, dw, ws, stream);
        case 6: return launch_gw_n<6, TIn>(g, x, dy, dw, ws, stream);
        case 7: return launch_gw_n<7, TIn>(g, x, dy, dw, ws, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

const char* grad_kernel_name(const Geom& g, int which, int dtype)
{
    if (which == 1) {
        if (grad_narrow_supported(g, dtype)) return "ukst_grad_weight_narrow_kernel";
        GwB16Args ba;
        if (dtype == 1 && gw_b16_args(g, ba)) return "ukst_grad_weight_mfma_bf16_kernel";
        GwMfmaArgs wa;
        const bool m = g.n <= 4 ? gw_mfma_args<gw_nc(4)>(g, wa) : gw_mfma_args<gw_nc(5)>(g, wa);
        if (m) return "ukst_grad_weight_mfma_kernel";
        GwThinArgs ta;
        int MT = 1, CT = 1;
        const bool th = g.n == 2 ? gw_thin_pick<2>(g, ta, MT, CT) : g.n == 3 ? gw_thin_pick<3>(g, ta, MT, CT)
                      : g.n == 4 ? gw_thin_pick<4>(g, ta, MT, CT) : g.n == 5 ? gw_thin_pick<5>(g, ta, MT, CT) : false;
        return th ? "ukst_grad_weight_thin_mfma_kernel" : "ukst_grad_weight_kernel";
    }
    if (grad_input_window_supported(g, dtype)) return "ukst_grad_input_window_mfma_bf16_kernel";
    if (grad_narrow_supported(g, dtype)) return "ukst_grad_input_narrow_kernel";
    GiMfmaArgs ma;
    if (dtype == 1 && gi_mfma_args(g, ma, true)) return "ukst_grad_input_mfma_bf16_kernel";
    return gi_mfma_args(g, ma) ? "ukst_grad_input_mfma_kernel" : "ukst_grad_input_kernel";
}

hipError_t launch_grad_input(const Geom& g, const void* dy, const void* w, float* dx, int dtype,
                             Workspace& ws, hipStream_t stream)
{
    switch (g.n) {
        case 1: return launch_gi_n<1>(g, dy, w, dx, dtype, ws, stream);
        case 2: return launch_gi_n<2>(g, dy, w, dx, dtype, ws, stream);
        case 3: return launch_gi_n<3>(g, dy, w, dx, dtype, ws, stream);
        case 4: return launch_gi_n<4>(g, dy, w, dx, dtype, ws, stream);
        case 5: return launch_gi_n<5>(g, dy, w, dx, dtype, ws, stream);
        case 6: return launch_gi_n<6>(g, dy, w, dx, dtype, ws, stream);
        case 7: return launch_gi_n<7>(g, dy, w, dx, dtype, ws, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_grad_weight(const Geom& g, const void* x, const void* dy, float* dw, int dtype,
                              Workspace& ws, hipStream_t stream)
{
    if (grad_narrow_supported(g, dtype)) return launch_grad_narrow(1, g, x, dy, dw, ws, stream);
    return dtype == 1 ? launch_gw_t<uint16_t>(g, x, dy, dw, ws, stream)
                      : launch_gw_t<float>(g, x, dy, dw, ws, stream);
}

}  // namespace ukst
