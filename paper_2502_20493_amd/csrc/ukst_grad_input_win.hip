// Gradient with respect to the input for bf16 operands and 4 x 4 kernels, on the bf16 matrix pipe
// with the taps inside the contraction.
//
// Differentiating Eqs. 1-4 gives dx[b,ci,i,j] = sum_co sum_{k,l} dy[b,co,2i+P-k,2j+P-l] w[co,ci,k,l]:
// a stride-2 convolution of dy with the kernel, in which every tap meets data (no inserted zeros
// exist on this side).  With kr = 3-k, lr = 3-l the 16 taps of one output channel are a 4 x 4
// window of dy that starts at (2i+P-3, 2j+P-3), and 16 is the K extent of
// v_mfma_f32_32x32x16_bf16.  One instruction therefore takes one output channel:
//   A (rows = input channels): lane (ci, kk) holds w[co][ci] for kr in {2kk, 2kk+1}, lr = 0..3 --
//     16 contiguous bytes of the weights packed once per call as [ci tile][co][kk][ci][8];
//   B (columns = pixels): lane (pixel, kk) holds dy rows 2i+P-3+2kk and +1, columns 2j+P-3 .. +3 --
//     two 8-byte reads from a dy tile that sits in LDS exactly as it sits in memory.
// Nothing is transposed or parity-split on the way in: staging is a copy (16-byte pieces, the tile
// origin at an even LDS element so that the window reads are 4-byte aligned; pieces that straddle
// an end of their dy row are fetched from inside the row and shifted into place).
//
// Block = 4 waves, tile = 128 input channels x 512 pixels ((image, row) pairs x TJ columns); a wave
// owns all 128 channels of 128 pixels: 16 accumulator tiles in 256 accumulation registers, one wave
// per SIMD.  A stage is 8 output channels (8 x 16 MFMAs per wave); both operands are double
// buffered in LDS and the next stage's pieces are written, and the registers refilled for the
// stage after next, one item after one MFMA, so that the matrix pipe never waits for staging.
#include "ukst_internal.h"

namespace ukst {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2a4 __attribute__((ext_vector_type(2), aligned(4)));
typedef unsigned u32x4a2 __attribute__((ext_vector_type(4), aligned(2)));
constexpr unsigned kInvalid = 0xFFFFFF00u;  // byte offset that is out of range for any buffer
constexpr int kRsrcFlags = 0x00020000;      // raw 32-bit buffer, gfx9 family

constexpr int CI_T = 128;                         // input channels per block
constexpr int KC = 8;                             // output channels per stage
constexpr int PIX = 512;                          // pixels per block
constexpr int A_BYTES = KC * 2 * CI_T * 16;       // weights of a stage: [co][kk][ci][8] bf16
constexpr int NPA = A_BYTES / 16 / 256;           // 16-byte weight pieces per thread and stage
constexpr int NPB = 12;                           // dy pieces per thread and stage, at most
constexpr int NIT = NPA + NPB;                    // staging items per thread and stage
constexpr int IPS = 3;                            // items dealt to a multiplication step (steps 0..6)
static_assert(NIT <= 7 * IPS, "items must fit the steps before the barrier");

struct GiWinArgs {
    GeomBase g;
    int TJ, logTJ, TI, logTI, TB;
    int LR;                    // staged dy rows per image: 2 TI + 2
    int S;                     // bytes per staged dy row
    int c8;                    // 16-byte pieces per staged dy row
    int rows;                  // staged dy rows per channel: TB * LR
    int coBytes;               // rows * S
    int bBytes;                // dy bytes of a stage in LDS, with the 16 spare bytes absent pieces go to
    int tilesX, tilesY, tilesB, ciTiles;
    int nStages;
};

// The value, through an empty statement the compiler cannot see through: sums of a per-thread base
// and a (buffer, step) offset are then formed where they are used, not kept in registers for every
// combination (which spills).
__device__ __forceinline__ int opaque(int v)
{
    asm volatile("" : "+v"(v));
    return v;
}

// wp[cit][co][kk][ci % 128][e]: tap (kr, lr) = (2 kk + e / 4, e % 4) is w[co][ci][3 - kr][3 - lr]
__global__ __launch_bounds__(256) void ukst_pack_w_window_kernel(const uint16_t* __restrict__ w,
                                                                uint16_t* __restrict__ wp, int Cout, int Cin,
                                                                int CIp)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)CIp * Cout * 16) return;
    const int e = (int)(idx & 7);
    const int cil = (int)((idx >> 3) & (CI_T - 1));
    const int kk = (int)((idx >> 10) & 1);
    const size_t r = idx >> 11;
    const int co = (int)(r % Cout), cit = (int)(r / Cout);
    const int ci = cit * CI_T + cil;
    const int kr = 2 * kk + (e >> 2), lr = e & 3;
    wp[idx] = ci < Cin ? w[((size_t)co * Cin + ci) * 16 + (3 - kr) * 4 + (3 - lr)] : (uint16_t)0;
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void ukst_grad_input_window_bf16_kernel(const uint16_t* __restrict__ dy,
                                                                            const uint16_t* __restrict__ wp,
                                                                            float* __restrict__ dx, GiWinArgs a)
{
    extern __shared__ __align__(16) unsigned char lds[];  // A[2][A_BYTES], then B[2][bBytes]
    const GeomBase& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kk = lane >> 5;
    const int tid16 = 16 * tid;

    int bid = xcd_contiguous(blockIdx.x, gridDim.x);  // neighbours in this numbering share an L2
    const int cit = bid % a.ciTiles; bid /= a.ciTiles;
    const int tx = bid % a.tilesX; bid /= a.tilesX;
    const int ty = bid % a.tilesY; bid /= a.tilesY;
    const int b0 = bid * a.TB, i0 = ty * a.TI, j0 = tx * a.TJ, ci0 = cit * CI_T;
    const int oy_base = 2 * i0 + g.P - 3, ox_base = 2 * j0 + g.P - 3;
    const size_t plane = (size_t)g.OH * g.OW;

    // dy of the tile's images, and this channel tile's packed weights, as raw buffers
    const size_t img0 = (size_t)b0 * g.Cout * plane;
    const size_t left = ((size_t)g.B * g.Cout * plane - img0) * 2;
    const __amdgpu_buffer_rsrc_t rs_dy = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(dy + img0), 0, (int)(left < 0xFFFFFF00u ? left : 0xFFFFFF00u), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(wp + (size_t)cit * g.Cout * (2 * CI_T * 8)), 0, a.nStages * A_BYTES, kRsrcFlags);
    const unsigned co_stage_bytes = (unsigned)(KC * plane * 2);

    // this thread's dy pieces: global offset (channel 0 of a stage) and LDS offset.  A piece that
    // straddles an end of its dy row is fetched from the nearest position inside the row and written
    // to where those columns belong, 2-byte aligned (it rewrites part of its neighbour with the same
    // values); the columns outside the row are never written and keep the zeros of the first fill.
    unsigned b_voff[NPB];
    int b_loff[NPB];
    {
        const int npieces = KC * a.rows * a.c8;
#pragma unroll
        for (int u = 0; u < NPB; ++u) {
            const int e = tid + 256 * u;
            b_voff[u] = kInvalid; b_loff[u] = KC * a.coBytes;
            if (e < npieces) {
                const int row_all = e / a.c8, pc = e - row_all * a.c8;
                const int co_l = row_all / a.rows, rem = row_all - co_l * a.rows;
                const int bl = rem / a.LR, rr = rem - bl * a.LR;
                const int b = b0 + bl, oy = oy_base + rr, ox = ox_base + 8 * pc;
                int start = ox;
                if (b < g.B && oy >= 0 && oy < g.OH && ox + 7 >= 0 && ox < g.OW) {
                    start = ox < 0 ? 0 : (ox + 8 > g.OW ? g.OW - 8 : ox);
                    b_voff[u] = (unsigned)((((size_t)bl * g.Cout + co_l) * plane + (size_t)oy * g.OW + start) * 2);
                }
                b_loff[u] = co_l * a.coBytes + rem * a.S + 2 * (start - ox_base);
            }
        }
    }

    u32x4 R[NIT];
    auto load_item = [&](int it, int stage) {
        if (it < NPA)
            R[it] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, (unsigned)tid16,
                                                          (unsigned)(stage * A_BYTES + 4096 * it), 0);
        else
            R[it] = __builtin_amdgcn_raw_buffer_load_b128(rs_dy, b_voff[it - NPA],
                                                          (unsigned)stage * co_stage_bytes, 0);
    };
    auto store_item = [&](int it, int buf) {
        if (it < NPA) {
            *reinterpret_cast<u32x4*>(lds + buf * A_BYTES + opaque(tid16) + 4096 * it) = R[it];
        } else {
            *reinterpret_cast<u32x4a2*>(lds + 2 * A_BYTES + buf * a.bBytes + opaque(b_loff[it - NPA])) = R[it];
        }
    };

    // window origin of this lane's pixel in each of the wave's four column tiles
    int boff[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int p = (wave * 4 + t) * 32 + l32;
        const int tr = p >> a.logTJ, lj = p & (a.TJ - 1);
        const int bl = tr >> a.logTI, li = tr & (a.TI - 1);
        boff[t] = 2 * A_BYTES + (bl * a.LR + 2 * li + 2 * kk) * a.S + 4 * lj;
    }
    const int aoff = (kk * CI_T + l32) * 16;

    bf16x8 fa[2][4], fb[2][4];
    auto load_fa = [&](int buf, int k, int slot, int mi) {
        fa[slot][mi] = *reinterpret_cast<const bf16x8*>(lds + buf * A_BYTES + k * (2 * CI_T * 16) + opaque(aoff) + mi * 512);
    };
    auto load_fb = [&](int buf, int k, int slot, int t) {
        const unsigned char* p = lds + opaque(boff[t]) + (buf * a.bBytes + k * a.coBytes);
        const u32x2a4 lo = *reinterpret_cast<const u32x2a4*>(p);
        const u32x2a4 hi = *reinterpret_cast<const u32x2a4*>(p + a.S);
        fb[slot][t] = __builtin_bit_cast(bf16x8, u32x4{lo.x, lo.y, hi.x, hi.y});
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][t][i] = 0.f;

    const int ns = a.nStages;
    // stage 0 into buffer 0, stage 1 into the registers
#pragma unroll
    for (int it = 0; it < NIT; ++it) load_item(it, 0);
    for (int o = tid16; o < 2 * a.bBytes; o += 4096)
        *reinterpret_cast<u32x4*>(lds + 2 * A_BYTES + o) = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();
#pragma unroll
    for (int it = 0; it < NIT; ++it) store_item(it, 0);
#pragma unroll
    for (int it = 0; it < NIT; ++it) load_item(it, ns > 1 ? 1 : 0);
    __syncthreads();
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) load_fa(0, 0, 0, mi);
#pragma unroll
    for (int t = 0; t < 4; ++t) load_fb(0, 0, 0, t);

    // one stage: 8 steps of 16 MFMAs; after each MFMA one side operation (a fragment of the next
    // step, or one staging item: its data goes to the other buffer, its registers are refilled)
    auto stage = [&](auto buf_tag, int s) {
        constexpr int BUF = decltype(buf_tag)::value;
        const int s2 = s + 2 < ns ? s + 2 : ns - 1;
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            const int cur = k & 1, nxt = cur ^ 1;
            const int fbuf = k + 1 < KC ? BUF : BUF ^ 1, fk = k + 1 < KC ? k + 1 : 0;
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                const int mi = m >> 2, t = m & 3;
                if (k == KC - 1 && m == 0) {
                    // every wave has read its last fragments of this buffer and written the other one
                    __syncthreads();
                }
                acc[mi][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][mi], fb[cur][t], acc[mi][t], 0, 0, 0);
                if (m == 0) load_fa(fbuf, fk, nxt, 0);
                else if (m <= 4) load_fb(fbuf, fk, nxt, m - 1);
                else if (m <= 7) load_fa(fbuf, fk, nxt, m - 4);
                else if (k < KC - 1 && m - 8 < IPS) {
                    const int it = k * IPS + (m - 8);
                    if (it < NIT) { store_item(it, BUF ^ 1); load_item(it, s2); }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    const std::integral_constant<int, 0> t0;
    const std::integral_constant<int, 1> t1;
    for (int s = 0; s < ns; s += 2) {  // ns is even (a second stage under a condition of its own spills)
        stage(t0, s);
        stage(t1, s + 1);
    }

    // drain: lanes along the pixel columns, a lane's 16 values of a tile are 16 input channels
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int p = (wave * 4 + t) * 32 + l32;
        const int tr = p >> a.logTJ, lj = p & (a.TJ - 1);
        const int b = b0 + (tr >> a.logTI), i = i0 + (tr & (a.TI - 1)), j = j0 + lj;
        if (b >= g.B || i >= g.H || j >= g.W) continue;
        float* out = dx + (((size_t)b * g.Cin + ci0) * g.H + i) * g.W + j;
        const size_t cs = (size_t)g.H * g.W;
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int cl = mi * 32 + 8 * (r / 4) + 4 * kk + (r % 4);
                if (ci0 + cl < g.Cin) out[cl * cs] = acc[mi][t][r];
            }
    }
}

int log2_of(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }

// bank pressure of the window reads of one wave for a row stride of S bytes: dwords that share a
// bank with another dword of the same read, summed over the 64 banks
int window_conflicts(int S, int TJ)
{
    int count[64], extra = 0;
    for (int b = 0; b < 64; ++b) count[b] = 0;
    bool seen[4096] = {false};
    for (int lane = 0; lane < 64; ++lane) {
        const int l32 = lane & 31, kk = lane >> 5;
        const int lj = l32 & (TJ - 1), lsub = TJ >= 32 ? 0 : l32 / TJ;
        for (int d = 0; d < 2; ++d) {
            const int dw = ((2 * lsub + 2 * kk) * S + 4 * lj) / 4 + d;
            if (dw >= 4096 || seen[dw]) continue;
            seen[dw] = true;
            if (count[dw & 63]++ > 0) ++extra;
        }
    }
    return extra;
}

}  // namespace

static bool gi_win_args(const Geom& g, GiWinArgs& a)
{
    if (g.n != 4 || g.Cout % (2 * KC) != 0 || g.Cin <= 64 || g.W < 16 || g.OW < 8 || g.H < 1)
        return false;
    a.g = g;
    a.TJ = g.W <= 16 ? 16 : g.W <= 32 ? 32 : 64;
    a.logTJ = log2_of(a.TJ);
    const int TR = PIX / a.TJ;
    a.TI = 1 << log2_of(g.H < TR ? g.H : TR);
    a.logTI = log2_of(a.TI);
    a.TB = TR / a.TI;
    a.LR = 2 * a.TI + 2;
    a.rows = a.TB * a.LR;
    a.c8 = (2 * a.TJ + 2 + 7) / 8;
    if ((KC * a.rows * a.c8 + 255) / 256 > NPB) return false;
    // row stride: the smallest multiple of 16 bytes with the fewest bank clashes that still fits
    int best = -1, best_cost = 1 << 30;
    for (int m = 0; m <= 8; ++m) {
        const int S = 16 * (a.c8 + m);
        if (2 * (size_t)A_BYTES + 2 * ((size_t)KC * a.rows * S + 16) > 160 * 1024) break;
        const int c = window_conflicts(S, a.TJ);
        if (c < best_cost) { best_cost = c; best = S; }
    }
    if (best < 0) return false;
    a.S = best;
    a.coBytes = a.rows * a.S;
    a.bBytes = KC * a.coBytes + 16;
    a.tilesX = (g.W + a.TJ - 1) / a.TJ;
    a.tilesY = (g.H + a.TI - 1) / a.TI;
    a.tilesB = (g.B + a.TB - 1) / a.TB;
    a.ciTiles = (g.Cin + CI_T - 1) / CI_T;
    a.nStages = g.Cout / KC;
    // a piece moved back inside its row must not start before its tile's first column
    if (2 * (a.tilesX - 1) * a.TJ + g.P - 3 + 8 > g.OW) return false;
    const size_t plane = (size_t)g.OH * g.OW;
    // offsets inside a tile's images and inside a channel tile's weights stay below the invalid mark
    if ((size_t)a.TB * g.Cout * plane * 2 + 64 >= 0xFFFFFF00u) return false;
    if ((size_t)a.nStages * A_BYTES >= 0x7FFFFFFFu) return false;
    if ((long long)a.tilesX * a.tilesY * a.tilesB * a.ciTiles > 0x7fffffffLL) return false;
    return true;
}

bool grad_input_window_supported(const Geom& g, int dtype)
{
    GiWinArgs a;
    return dtype == 1 && gi_win_args(g, a);
}

hipError_t launch_grad_input_window(const Geom& g, const void* dy, const void* w, float* dx, Workspace& ws,
                                    hipStream_t stream)
{
    GiWinArgs a;
    if (!gi_win_args(g, a)) return hipErrorInvalidValue;
    const size_t pelems = (size_t)a.ciTiles * CI_T * g.Cout * 16;
    const size_t need = ws_align(pelems * 2);
    if (ws.query) { ws.need = need; return hipSuccess; }
    if (ws.bytes < need) return kWorkspaceTooSmall;
    uint16_t* wp = (uint16_t*)ws.ptr;
    hipLaunchKernelGGL(ukst_pack_w_window_kernel, dim3((unsigned)((pelems + 255) / 256)), dim3(256), 0, stream,
                       (const uint16_t*)w, wp, g.Cout, g.Cin, a.ciTiles * CI_T);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t lds = 2 * (size_t)A_BYTES + 2 * (size_t)a.bBytes;
    e = hipFuncSetAttribute((const void*)ukst_grad_input_window_bf16_kernel,
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const unsigned nb = (unsigned)((long long)a.tilesX * a.tilesY * a.tilesB * a.ciTiles);
    hipLaunchKernelGGL(ukst_grad_input_window_bf16_kernel, dim3(nb), dim3(256), lds, stream,
                       (const uint16_t*)dy, (const uint16_t*)wp, dx, a);
    return hipGetLastError();
}

}  // namespace ukst
