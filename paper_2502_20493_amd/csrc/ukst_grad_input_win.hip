// Gradient with respect to the input for bf16 operands and kernels of up to 4 x 4, on the bf16
// matrix pipe with the taps inside the contraction.  (Written for n = 4 below; a smaller kernel sits
// in the same 4 x 4 frame, which then starts at (2i+P-(n-1), 2j+P-(n-1)) and has zero weights in its
// last 4-n rows and columns: 9 (n = 3) or 4 (n = 2) of the 16 K slots do useful work, which is still
// twice as fast as transposing dy.  A dy value that is not finite therefore also reaches the input
// pixels whose frames hold it in a zero-weight slot.)
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
// origin at an even LDS element so that the window reads are 4-byte aligned; a piece that hangs
// over an end of its dy row is fetched from inside the row and written where those columns belong,
// at a 2-byte-aligned LDS address).
//
// Block = 4 waves, tile = 128 input channels x 512 pixels ((image, row) pairs x TJ columns); a wave
// owns all 128 channels of 128 pixels: 16 accumulator tiles in 256 accumulation registers, one wave
// per SIMD.  A stage is 8 output channels (8 x 16 MFMAs per wave); both operands are double
// buffered in LDS and the next stage's pieces are written, and the registers refilled for the
// stage after next, one item after one MFMA.  Blocks are persistent: one per compute unit, each
// walking over every gridDim.x-th tile with the staging pipeline running on into the next tile.
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
    int tilesX, tilesY, tilesB, ciTiles, nTiles;
    int nStages;
    FastDiv dC8, dRows, dLR;
};

// The value, through an empty statement the compiler cannot see through: sums of a per-thread base
// and a (buffer, step) offset are then formed where they are used, not kept in registers for every
// combination (which spills).
__device__ __forceinline__ int opaque(int v)
{
    asm volatile("" : "+v"(v));
    return v;
}

// wp[cit][co][kk][ci % 128][e]: slot (kr, lr) = (2 kk + e / 4, e % 4) of the 4 x 4 frame is
// w[co][ci][n-1-kr][n-1-lr], zero where that tap does not exist (n < 4: the last frame rows and columns)
__global__ __launch_bounds__(256) void ukst_pack_w_window_kernel(const uint16_t* __restrict__ w,
                                                                uint16_t* __restrict__ wp, int Cout, int Cin,
                                                                int CIp, int n)
{
    // one thread per 16-byte piece: the eight slots e of (cit, co, kk, ci)
    const size_t piece = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (piece >= (size_t)CIp * Cout * 2) return;
    const int cil = (int)(piece & (CI_T - 1));
    const int kk = (int)((piece >> 7) & 1);
    const size_t r = piece >> 8;
    const int co = (int)(r % Cout), cit = (int)(r / Cout);
    const int ci = cit * CI_T + cil;
    u32x4 out = {0u, 0u, 0u, 0u};
    if (ci < Cin) {
        const uint16_t* src = w + ((size_t)co * Cin + ci) * (n * n);
        if (n == 4) {
            // slots 8 kk .. 8 kk + 7 are taps 15 - 8 kk down to 8 - 8 kk: eight consecutive taps, reversed
            const u32x4a2 q = *reinterpret_cast<const u32x4a2*>(src + 8 * (1 - kk));
            const unsigned t[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) out[j] = __builtin_amdgcn_alignbit(t[3 - j], t[3 - j], 16);  // halves swapped
        } else {
            unsigned h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = n - 1 - (2 * kk + (e >> 2)), l = n - 1 - (e & 3);
                h[e] = k >= 0 && l >= 0 ? src[k * n + l] : 0u;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) out[j] = h[2 * j] | (h[2 * j + 1] << 16);
        }
    }
    *reinterpret_cast<u32x4*>(wp + piece * 8) = out;
}

template <int SD>  // dwords per staged dy row
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void ukst_grad_input_window_mfma_bf16_kernel(const uint16_t* __restrict__ dy, const uint16_t* __restrict__ wp,
                                        float* __restrict__ dx, GiWinArgs a)
{
    constexpr int S = 4 * SD;
    extern __shared__ __align__(16) unsigned char lds[];  // A[2][A_BYTES], then B[2][bBytes]
    const GeomBase& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kk = lane >> 5;
    const int tid16 = 16 * tid;
    const size_t plane = (size_t)g.OH * g.OW;
    const unsigned co_stage_bytes = (unsigned)(KC * plane * 2);
    const int nreal = a.nStages;          // stages of 8 output channels that exist
    const int ns = (nreal + 1) & ~1;      // an odd count is padded with a stage of zeros
    const int G = gridDim.x;

    // tile of a position in the walk: channel tile fastest, so that the blocks of one XCD (which
    // take neighbouring positions) read the same dy through one L2
    struct Tile { int cit, tx, b0, i0, j0; };
    auto tile_at = [&](int lin) {
        Tile t;
        t.cit = lin % a.ciTiles; lin /= a.ciTiles;
        t.tx = lin % a.tilesX; lin /= a.tilesX;
        const int ty = lin % a.tilesY; lin /= a.tilesY;
        t.b0 = lin * a.TB; t.i0 = ty * a.TI; t.j0 = t.tx * a.TJ;
        return t;
    };

    // Load side of the staging pipeline (it runs two stages ahead and therefore moves to the next
    // tile two stages early): dy of the tile's images and the channel tile's packed weights as raw
    // buffers, and this thread's dy pieces as byte offsets of channel 0 of a stage.  A piece that
    // straddles an end of its dy row is fetched from the nearest position inside the row and
    // written to where those columns belong, 2-byte aligned (it rewrites part of its neighbour
    // with the same values); columns outside the row are never written and stay zero.
    __amdgpu_buffer_rsrc_t rs_dy, rs_w;
    unsigned a_voff, b_voff[NPB];
    int b_loff[NPB];  // LDS address of the piece in the buffer written next
    const int npieces = KC * a.rows * a.c8;
    auto piece_start = [&](int ox) {  // first column fetched for the piece that begins at column ox
        return (ox < 0 && ox + 7 >= 0) ? 0 : (ox < g.OW && ox + 8 > g.OW) ? g.OW - 8 : ox;
    };
    auto aim_loads = [&](const Tile& t, bool present) {
        const size_t img0 = (size_t)t.b0 * g.Cout * plane;
        const size_t left = ((size_t)g.B * g.Cout * plane - img0) * 2;
        rs_dy = __builtin_amdgcn_make_buffer_rsrc((void*)(dy + img0), 0,
                                                  (int)(left < 0xFFFFFF00u ? left : 0xFFFFFF00u), kRsrcFlags);
        rs_w = __builtin_amdgcn_make_buffer_rsrc((void*)(wp + (size_t)t.cit * g.Cout * (2 * CI_T * 8)), 0,
                                                 nreal * A_BYTES, kRsrcFlags);
        a_voff = present ? (unsigned)tid16 : kInvalid;
        const int oy_base = 2 * t.i0 + g.P - (g.n - 1), ox_base = 2 * t.j0 + g.P - (g.n - 1);
        const int tid_o = opaque(tid);  // nothing of this is to be kept from tile to tile
#pragma unroll
        for (int u = 0; u < NPB; ++u) {
            const int e = tid_o + 256 * u;
            b_voff[u] = kInvalid;
            if (present && e < npieces) {
                const int row_all = fdiv(e, a.dC8), pc = e - row_all * a.c8;
                const int co_l = fdiv(row_all, a.dRows), rem = row_all - co_l * a.rows;
                const int bl = fdiv(rem, a.dLR), rr = rem - bl * a.LR;
                const int b = t.b0 + bl, oy = oy_base + rr, ox = ox_base + 8 * pc;
                if (b < g.B && oy >= 0 && oy < g.OH && ox + 7 >= 0 && ox < g.OW)
                    b_voff[u] = (unsigned)((((size_t)bl * g.Cout + co_l) * plane + (size_t)oy * g.OW +
                                            piece_start(ox)) * 2);
            }
        }
    };
    // Store side: where the pieces go in buffer `buf` (depends on the tile's columns only)
    auto aim_stores = [&](const Tile& t, int buf) {
        const int ox_base = 2 * t.j0 + g.P - (g.n - 1);
        const int tid_o = opaque(tid);
#pragma unroll
        for (int u = 0; u < NPB; ++u) {
            const int e = tid_o + 256 * u;
            b_loff[u] = 2 * A_BYTES + buf * a.bBytes + KC * a.coBytes;  // the spare 16 bytes
            if (e < npieces) {
                const int row_all = fdiv(e, a.dC8), pc = e - row_all * a.c8;
                const int ox = ox_base + 8 * pc;
                b_loff[u] = 2 * A_BYTES + buf * a.bBytes + row_all * S + 2 * (piece_start(ox) - ox_base);
            }
        }
    };
    auto zero_fill = [&](int buf) {
        for (int o = tid16; o < a.bBytes; o += 4096)
            *reinterpret_cast<u32x4*>(lds + 2 * A_BYTES + buf * a.bBytes + o) = u32x4{0u, 0u, 0u, 0u};
    };

    u32x4 R[NIT];
    auto load_item = [&](int it, int stage) {
        const bool real = stage < nreal;  // uniform; the padding stage reads zeros through the invalid offset
        if (it < NPA)
            R[it] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, real ? a_voff : kInvalid,
                                                          real ? (unsigned)(stage * A_BYTES + 4096 * it) : 0u, 0);
        else
            R[it] = __builtin_amdgcn_raw_buffer_load_b128(rs_dy, real ? b_voff[it - NPA] : kInvalid,
                                                          real ? (unsigned)stage * co_stage_bytes : 0u, 0);
    };
    // writes the item into buffer `buf`; dtoggle turns its LDS address to the other buffer afterwards
    auto store_item = [&](int it, int buf, int dtoggle) {
        if (it < NPA) {
            *reinterpret_cast<u32x4*>(lds + tid16 + (buf * A_BYTES + 4096 * it)) = R[it];
        } else {
            *reinterpret_cast<u32x4a2*>(lds + b_loff[it - NPA]) = R[it];
            b_loff[it - NPA] += dtoggle;
        }
    };

    // window origin of this lane's pixel in each of the wave's four column tiles (buffer 0, channel 0)
    int boff[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int p = (wave * 4 + t) * 32 + l32;
        const int tr = p >> a.logTJ, lj = p & (a.TJ - 1);
        const int bl = tr >> a.logTI, li = tr & (a.TI - 1);
        boff[t] = 2 * A_BYTES + (bl * a.LR + 2 * li + 2 * kk) * S + 4 * lj;
    }
    const int aoff = (kk * CI_T + l32) * 16;

    bf16x8 fa[4], fb[2][4];  // weights: one set, each reloaded right after its last use in a step
    int bp[4];  // LDS address of the window rows the next B fragment is read from
    auto load_fa = [&](int buf, int k, int mi) {
        fa[mi] = *reinterpret_cast<const bf16x8*>(lds + aoff + (buf * A_BYTES + k * (2 * CI_T * 16) + mi * 512));
    };
    auto load_fb = [&](int slot, int t, int advance) {
        const unsigned char* p = lds + bp[t];
        const u32x2a4 lo = *reinterpret_cast<const u32x2a4*>(p);
        const u32x2a4 hi = *reinterpret_cast<const u32x2a4*>(p + S);
        fb[slot][t] = __builtin_bit_cast(bf16x8, u32x4{lo.x, lo.y, hi.x, hi.y});
        bp[t] += advance;
    };

    int lin = xcd_contiguous(blockIdx.x, G);
    Tile cur = tile_at(lin);

    // first tile: zeros everywhere, stage 0 into buffer 0, stage 1 into the registers
    aim_loads(cur, true);
    aim_stores(cur, 0);
#pragma unroll
    for (int it = 0; it < NIT; ++it) load_item(it, 0);
    zero_fill(0);
    zero_fill(1);
    __syncthreads();
#pragma unroll
    for (int it = 0; it < NIT; ++it) store_item(it, 0, a.bBytes);
#pragma unroll
    for (int it = 0; it < NIT; ++it) load_item(it, 1);
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 4; ++t) bp[t] = boff[t];
#pragma unroll
    for (int mi = 0; mi < 3; ++mi) load_fa(0, 0, mi);
#pragma unroll
    for (int t = 0; t < 4; ++t) load_fb(0, t, a.coBytes);

    const std::integral_constant<int, 0> t0;
    const std::integral_constant<int, 1> t1;
    bool stale1 = false;  // buffer 1 still holds columns of a tile whose rows ended elsewhere
    for (;;) {
        const int nlin = lin + G;
        const bool more = nlin < a.nTiles;  // uniform
        const Tile nxt = tile_at(more ? nlin : lin);
        const bool refill = more && nxt.tx != cur.tx;  // the next tile's rows end at other LDS columns

        f32x16 acc[4][4];
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[mi][t][i] = 0.f;

        // one stage: 8 steps of 16 MFMAs; after an MFMA at most one side operation (a fragment of
        // the next step, or one staging item: its data goes to the other buffer, its registers are
        // refilled for the stage after next)
        auto stage = [&](auto buf_tag, int s) {
            constexpr int BUF = decltype(buf_tag)::value;
            if constexpr (BUF == 0) {
                if (s == 0 && stale1) {
                    zero_fill(1);  // free since the last stage of the tile before
                    __syncthreads();
                }
                if (s == ns - 2) aim_loads(nxt, more);  // the loads of this stage are the next tile's first
            } else {
                if (s == ns - 1 && refill) {
                    // buffer 0 is free: its stale columns beside the next tile's rows go, then its pieces
                    zero_fill(0);
                    aim_stores(nxt, 0);
                    __syncthreads();
                }
            }
            const int s2 = s + 2 < ns ? s + 2 : s + 2 - ns;
            // values the compiler shall not trace through the stages (it would keep every sum of a
            // base and a (buffer, step) offset in a register of its own, and spill)
#pragma unroll
            for (int t = 0; t < 4; ++t) asm volatile("" : "+v"(bp[t]));
#pragma unroll
            for (int u = 0; u < NPB; ++u) asm volatile("" : "+v"(b_loff[u]));
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                const int cur_f = k & 1, nxt_f = cur_f ^ 1;
                const int fbuf = k + 1 < KC ? BUF : BUF ^ 1, fk = k + 1 < KC ? k + 1 : 0;
                // after this step's reads: one channel on; from channel 7 to channel 0 of the other buffer
                const int adv = k == KC - 2 ? (BUF == 0 ? a.bBytes : -a.bBytes) - (KC - 1) * a.coBytes : a.coBytes;
#pragma unroll
                for (int m = 0; m < 16; ++m) {
                    const int mi = m >> 2, t = m & 3;
                    if (k == KC - 1 && m == 1) {
                        // every wave has read its last fragments of this buffer and written the other one
                        __syncthreads();
                    }
                    acc[mi][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[cur_f][t], acc[mi][t], 0, 0, 0);
                    if (m == 0) load_fa(BUF, k, 3);                       // this step's last weights
                    else if (m <= 4) load_fb(nxt_f, m - 1, adv);
                    else if (m == 5) load_fa(fbuf, fk, 0);                // the next step's, as they fall free
                    else if (m == 8) load_fa(fbuf, fk, 1);
                    else if (m == 12) load_fa(fbuf, fk, 2);
                    else if (k < KC - 1 && (m == 6 || m == 7 || m == 9)) {
                        const int it = k * IPS + (m == 9 ? 2 : m - 6);
                        if (it < NIT) {
                            store_item(it, BUF ^ 1, BUF == 0 ? -a.bBytes : a.bBytes);
                            load_item(it, s2);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        for (int s = 0; s < ns; s += 2) {  // ns is even (a second stage call under a condition of its own spills)
            stage(t0, s);
            stage(t1, s + 1);
        }

        // drain: lanes along the pixel columns, a lane's 16 values of a tile are 16 input channels.
        // Raw buffer stores: the pixel (and the lane's half of the channel octet) is the vector
        // offset, the channel the scalar offset; absent pixels carry the invalid offset and drop out.
        {
            const int ci0 = cur.cit * CI_T;
            const size_t cs = (size_t)g.H * g.W;
            const size_t base = ((size_t)cur.b0 * g.Cin + ci0) * cs;
            const size_t left = ((size_t)g.B * g.Cin * cs - base) * 4;
            const __amdgpu_buffer_rsrc_t rs_dx = __builtin_amdgcn_make_buffer_rsrc(
                (void*)(dx + base), 0, (int)(left < 0xFFFFFF00u ? left : 0xFFFFFF00u), kRsrcFlags);
            const unsigned cs4 = (unsigned)(cs * 4);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int p = (wave * 4 + t) * 32 + l32;
                const int tr = p >> a.logTJ, lj = p & (a.TJ - 1);
                const int bl = tr >> a.logTI, i = cur.i0 + (tr & (a.TI - 1)), j = cur.j0 + lj;
                const bool ok = cur.b0 + bl < g.B && i < g.H && j < g.W;
                const unsigned voff = ok ? (unsigned)(((size_t)bl * g.Cin * cs + (size_t)i * g.W + j) * 4) + 4 * kk * cs4
                                         : kInvalid;
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if (ci0 + mi * 32 + 8 * q >= g.Cin) continue;  // uniform: Cin is a multiple of 8
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            // element by value, through a register of its own: a bit cast applied to
                            // an element of a vector reads element 0
                            float v = acc[mi][t][4 * q + r];
                            asm volatile("" : "+v"(v));
                            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), rs_dx, voff,
                                                                  (unsigned)(mi * 32 + 8 * q + r) * cs4, 0);
                        }
                    }
            }
        }
        if (!more) break;
        lin = nlin;
        cur = nxt;
        stale1 = refill;
    }
}

int log2_of(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }

}  // namespace

static bool gi_win_args(const Geom& g, GiWinArgs& a)
{
    if (g.n < 2 || g.n > 4 || g.Cout % KC != 0 || g.Cin <= 64 || g.Cin % 8 != 0 || g.W < 16 || g.OW < 8 || g.H < 1)
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
    // row stride: 2 S = 128 (mod 256) keeps the two row pairs of a window read in different banks;
    // 16-column tiles need 2 S = 96 (mod 128) for their two pixel rows per read
    const int cand[3][2] = {{80, 80}, {192, 160}, {320, 320}};
    int best = -1;
    for (int c = 0; c < 2 && best < 0; ++c) {
        const int S = cand[a.logTJ - 4][c];
        if (S >= 16 * a.c8 && 2 * (size_t)A_BYTES + 2 * ((size_t)KC * a.rows * S + 16) <= 160 * 1024) best = S;
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
    a.dC8 = make_fastdiv((unsigned)a.c8);
    a.dRows = make_fastdiv((unsigned)a.rows);
    a.dLR = make_fastdiv((unsigned)a.LR);
    // a piece moved back inside its row must not start before its tile's first column
    if (2 * (a.tilesX - 1) * a.TJ + g.P - (g.n - 1) + 8 > g.OW) return false;
    const size_t plane = (size_t)g.OH * g.OW;
    // offsets inside a tile's images and inside a channel tile's weights stay below the invalid mark
    if ((size_t)a.TB * g.Cout * plane * 2 + 64 >= 0xFFFFFF00u) return false;
    if ((size_t)a.nStages * A_BYTES >= 0x7FFFFFFFu) return false;
    if ((size_t)a.TB * g.Cin * g.H * g.W * 4 + 64 >= 0xFFFFFF00u) return false;
    const long long nt = (long long)a.tilesX * a.tilesY * a.tilesB * a.ciTiles;
    if (nt > 0x3fffffffLL) return false;
    a.nTiles = (int)nt;
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
    hipLaunchKernelGGL(ukst_pack_w_window_kernel, dim3((unsigned)((pelems / 8 + 255) / 256)), dim3(256), 0, stream,
                       (const uint16_t*)w, wp, g.Cout, g.Cin, a.ciTiles * CI_T, g.n);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t lds = 2 * (size_t)A_BYTES + 2 * (size_t)a.bBytes;
    typedef void (*kernel_t)(const uint16_t*, const uint16_t*, float*, GiWinArgs);
    const kernel_t kfn = a.S == 80 ? ukst_grad_input_window_mfma_bf16_kernel<20>
                       : a.S == 160 ? ukst_grad_input_window_mfma_bf16_kernel<40>
                       : a.S == 192 ? ukst_grad_input_window_mfma_bf16_kernel<48>
                                    : ukst_grad_input_window_mfma_bf16_kernel<80>;
    e = hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    // one block per compute unit (its LDS holds one), each walking over every cus-th tile
    int dev = 0, cus = 0;
    e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    const unsigned nb = (unsigned)(a.nTiles < cus ? a.nTiles : cus);
    hipLaunchKernelGGL(kfn, dim3(nb), dim3(256), lds, stream, (const uint16_t*)dy, (const uint16_t*)wp, dx, a);
    return hipGetLastError();
}

}  // namespace ukst
