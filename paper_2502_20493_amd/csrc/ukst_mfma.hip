// MFMA path: parity-class implicit GEMM on the matrix cores for wide layers.
//
// GEMM view (per quad, see ukst_internal.h): the four parity classes of a quad read the SAME
// ceil(n/2) x ceil(n/2) input window, so for window position (u, v) and input channel ci the
// activation x[ci][k-P+u][m-P+v] is one B operand shared by every class, and class (r, s)
// multiplies it by its own sub-kernel tap w[co][ci][r+2u][s+2v] (Eqs. 1-4).  Hence
//
//     D_rs[co][quad] += sum_ci  W_tap(r,s,u,v)[co][ci] * X_(u,v)[ci][quad]
//
// i.e. one MFMA B fragment feeds up to four MFMAs (one per class), and the kernel's n*n taps are
// each used once per quad (Sec. 3.1).  M = output channels, N = quads (flattened over batch, quad
// rows and quad columns so that tiles stay full whatever the image size), K = input channels.
// Lanes of an accumulator tile run along N = consecutive quad columns, so the epilogue writes the
// two column classes of a quad as one 8-byte store and a wave covers runs of 64 consecutive
// floats of an output row: the classes are interleaved in place, there is no re-arrangement pass
// and no second copy of the output (the cost Sec. 5 attributes to a GEMM formulation).
//
// Block = 256 threads = 4 waves; block tile = 64 output channels x 256 quads x 4 classes; wave
// tile = 32 channels x 128 quads x 4 classes = 16 accumulator tiles of 32x32 (256 registers).
// Blocks are persistent: one block per compute unit walks over tiles, and the K pipeline runs
// across tile boundaries (while the last stages of a tile are multiplied, the first stages of
// the next tile are already being fetched and laid out in LDS), so only the accumulator drain
// sits between two tiles.
// K advances 16 input channels per stage; stages are double-buffered in LDS: while the matrix
// cores work on stage s the global loads of stage s+2 are in flight.  NCHW keeps the K axis (ci)
// slowest, while an MFMA lane wants 8 consecutive K values in one register group: both operands
// are transposed in registers (8x8 b16 transposes out of v_perm_b32) on their way into LDS, which
// is where the sub-kernels get gathered per tap.
#include "ukst_internal.h"

namespace ukst {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned u2v __attribute__((ext_vector_type(2)));
typedef unsigned u4v __attribute__((ext_vector_type(4)));
typedef const float __attribute__((address_space(4)))* bias_cptr;

constexpr int kRsrcFlags = 0x00020000;      // raw 32-bit buffer, gfx9 family
constexpr unsigned kInvalid = 0xFFFFFF00u;  // byte offset that is out of range for any buffer

constexpr int TM = 64;    // output channels per block
constexpr int TN = 256;   // quads per block
constexpr int KC = 16;    // input channels per stage (one MFMA K step)
constexpr int W_PLANE = (TM + 1) * 16;  // bytes of one tap plane of a k-half (64 channels + 1 pad slot)
constexpr int W_HALF = 16 * W_PLANE + 64;  // bytes of one k-half (16 tap planes), skewed by 4 slots
constexpr int XS_STAGE_MAX = 40960;     // bytes reserved per activation stage buffer

struct MfmaArgs {
    GeomBase g;
    int Q;        // total quads = B * KH * KW
    int EH;       // distinct input rows one image's quad rows touch = KH + ceil(n/2) - 1
    int ROWS;     // input rows an activation stage buffer holds
    int LWS;      // 16-byte slots per staged row (columns + one pad slot per 8 + halo)
    int OFFS;     // LDS column of input column 0 (multiple of 8, >= floor(P/2))
    int C8;       // 8-column groups per input row
    int nco;      // channel blocks
    int nqt;      // quad tiles
    int ntiles;   // nco * nqt
    int cb_major; // tile order: 1 = consecutive tiles share the channel block (big weights),
                  //             0 = consecutive tiles share the quad tile (big activations)
    FastDiv dKHW, dKW, dEH, dC8, dROWS, dNCO, dNQT;
};

// 8x8 transpose of 16-bit elements held as 8 rows of 4 dwords: row k of the result collects
// element k of every input row.
__device__ __forceinline__ u4v transposed_row(const u4v (&in)[8], int k)
{
    u4v t;
    const int q = k >> 1;
    const unsigned sel = (k & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
    for (int pp = 0; pp < 4; ++pp) t[pp] = __builtin_amdgcn_perm(in[2 * pp + 1][q], in[2 * pp][q], sel);
    return t;
}

// The MFMA groups of a K step: one group = one parity class c = 2r + s at one window position
// p = u * HI + v that holds a tap for it, w[r + 2u][s + 2v] (Eqs. 1-4): 16 groups for n = 4 (every
// class has 2 x 2 taps), 9 for n = 3 (4 / 2 / 2 / 1 taps: the classes of Sec. 3.2 with unequal
// sub-kernels).  Groups are ordered by window position so that a B fragment is fetched once.
constexpr bool grp_valid(int n, int p, int c)
{
    const int hi = (n + 1) / 2, u = p / hi, v = p % hi, r = c >> 1, sc = c & 1;
    return r + 2 * u < n && sc + 2 * v < n;
}
constexpr int grp_count(int n)
{
    const int hi = (n + 1) / 2;
    int k = 0;
    for (int p = 0; p < hi * hi; ++p)
        for (int c = 0; c < 4; ++c) k += grp_valid(n, p, c) ? 1 : 0;
    return k;
}
// group gi -> p * 4 + c
constexpr int grp_at(int n, int gi)
{
    const int hi = (n + 1) / 2;
    int k = 0;
    for (int p = 0; p < hi * hi; ++p)
        for (int c = 0; c < 4; ++c)
            if (grp_valid(n, p, c)) {
                if (k == gi) return p * 4 + c;
                ++k;
            }
    return -1;
}
// how many groups of the same window position come before group gi
constexpr int grp_rank(int n, int gi)
{
    const int p = grp_at(n, gi) >> 2;
    int k = 0;
    for (int j = 0; j < gi; ++j) k += (grp_at(n, j) >> 2) == p ? 1 : 0;
    return k;
}

// EPI: the fused epilogue (bias, activation) is compiled into the drain; the plain instance keeps
// the register allocation of its drain to itself.  OUT16: y is bf16, each sum rounded once (to
// nearest even) at the store, the two column classes of a quad packed into one 4-byte store.
template <int N, bool EPI, bool OUT16>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void ukst_mfma_bf16_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
                           void* __restrict__ y, MfmaArgs a, Epilogue ep)
{
    static_assert(N == 4 || N == 3, "bf16 MFMA path: the in-register sub-kernel gather handles 9 or 16 taps");
    constexpr int HI = (N + 1) / 2;
    constexpr int NN = N * N;
    constexpr int WS_STAGE = 2 * W_HALF;  // 33408 bytes: [k-half][tap][channel][8 ci]
    extern __shared__ __align__(16) unsigned char lds[];
    // layout: weights stage 0, weights stage 1, activations stage 0, activations stage 1
    constexpr int XS_OFF = 2 * WS_STAGE;

    const GeomBase& g = a.g;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cw = wave & 1;   // which 32-channel half of the block tile
    const int qh = wave >> 1;  // which 128-quad half of the block tile
    const int l32 = lane & 31, gk = lane >> 5;
    const int KHW = g.KH * g.KW;
    const int G = gridDim.x;

    // Tile walked in round rho by this block.  Blocks are spread over the 8 XCDs round-robin, so
    // within a round the blocks of one XCD get 32 consecutive tile numbers: the tiles that share
    // weights or activations meet in the same L2 at the same time.
    const int xcd_rank = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);  // G is a multiple of 8
    auto tile_of = [&](int rho, int& cb, int& qt) -> bool {
        const int t = rho * G + xcd_rank;
        if (t >= a.ntiles) return false;
        // (both orders through the same assignments: a store to "cb or qt" picked by the flag
        // would put the two in scratch memory, and every later read behind all loads in flight)
        const int major = a.cb_major ? fdiv(t, a.dNQT) : fdiv(t, a.dNCO);
        const int minor = t - major * (a.cb_major ? a.nqt : a.nco);
        cb = a.cb_major ? major : minor;
        qt = a.cb_major ? minor : major;
        return true;
    };

    // ---- zero the activation buffers once: halo columns are never written again
    {
        const int n16 = 2 * XS_STAGE_MAX / 16;
        u4v z = {0u, 0u, 0u, 0u};
        for (int i = tid; i < n16; i += 256) *reinterpret_cast<u4v*>(lds + XS_OFF + i * 16) = z;
    }

    // ---- per-thread staging units
    // weights: thread = (channel co_l, k-half g, tap-half h), h fastest: the 8 loads of a thread
    // walk 8 input channels (32 bytes apart) and neighbouring lanes read neighbouring 16-byte
    // pieces, so every 64-byte line is consumed by consecutive instructions of one wave.  In LDS
    // the planes are skewed so that the 16 lanes of a write phase (4 channels x g x h) hit
    // distinct bank groups: co -> +1 slot, g -> +4 slots, h (8 planes) -> +8 slots (mod 16).
    const int w_co = tid >> 2, w_g = (tid >> 1) & 1, w_h = tid & 1;
    // n = 4: the tap-halves are taps 0-7 and 8-15.  n = 3 (9 taps, 18-byte rows, 16-byte loads at
    // 2-byte alignment): half 0 fetches taps 0-7, half 1 taps 1-8, whose rows go to planes 1-8 --
    // planes 1-7 are written twice with the same values, plane 8 is tap 8.
    constexpr int W_H_PLANES = N == 4 ? 8 : 1, W_H_BYTES = N == 4 ? 16 : 2;
    const int w_lds = w_g * W_HALF + (W_H_PLANES * w_h) * W_PLANE + w_co * 16;  // + t * W_PLANE
    // activations: thread = (8-column group c8, row r, k-half g), c8 fastest so that lanes walk
    // contiguous memory; threads beyond the unit count repeat a unit (same loads, same LDS
    // writes, no branch).  Column c sits in slot c + c/8: the pad slot after every 8 columns
    // spreads the 128-byte stride between neighbouring units over the LDS banks.
    int x_r, x_g, x_c8;
    {
        const int units = a.ROWS * 2 * a.C8;
        const int un = tid % units;
        const int t2 = fdiv(un, a.dC8);
        x_c8 = un - t2 * a.C8;
        x_g = fdiv(t2, a.dROWS);
        x_r = t2 - x_g * a.ROWS;
    }
    const int x_lds = ((x_g * a.ROWS + x_r) * a.LWS + (a.OFFS + 8 * x_c8) / 8 * 9) * 16;

    // global offsets of this thread's staging units for tile (cb, qt)
    auto staging_offsets = [&](int cb, int qt, unsigned& wv, unsigned& xv) {
        wv = cb * TM + w_co < g.Cout
                 ? (unsigned)(((cb * TM + w_co) * g.Cin + 8 * w_g) * (NN * 2) + w_h * W_H_BYTES)
                 : kInvalid;  // channels past the last one: zeros
        const int q0 = qt * TN;
        const int bf = fdiv(q0, a.dKHW), kf = fdiv(q0 - bf * KHW, a.dKW);
        const int e = bf * a.EH + kf + x_r;  // input row index over the whole batch
        const int b = fdiv(e, a.dEH), ii = e - b * a.EH;
        const int i = g.k_min - g.P + ii;
        xv = kInvalid;
        if (b < g.B && i >= 0 && i < g.H)
            xv = (unsigned)((((b * g.Cin + 8 * x_g) * g.H + i) * g.W + 8 * x_c8) * 2);
    };

    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
        (void*)x, 0, (int)((size_t)g.B * g.Cin * g.H * g.W * 2), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(
        (void*)w, 0, (int)((size_t)g.Cout * g.Cin * NN * 2), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(
        y, 0, (int)((size_t)g.B * g.Cout * g.OH * g.OW * (OUT16 ? 2 : 4)), kRsrcFlags);
    const unsigned x_cstride = (unsigned)(g.H * g.W * 2);  // bytes between input channels
    constexpr unsigned ES = OUT16 ? 2u : 4u;  // bytes per output element
    const unsigned plane = (unsigned)(g.OH * g.OW) * ES;

    // A (weights): lane = channel cw*32 + l32 of the block tile, k-half gk
    const int a_lds = gk * W_HALF + (cw * 32 + l32) * 16;

    // ---- software pipeline ----------------------------------------------------------------
    // Stage s lives in LDS buffer s&1 and passes through register set s&1.  Global loads are
    // requested two stages ahead of their use: one stage of MFMA work (64 x 8 passes) is shorter
    // than the memory latency under load.  Inside a stage every non-MFMA instruction is slotted
    // between groups of four MFMAs (one group = one parity class at one window position), so that
    // its issue time hides under the matrix pipe: per group one global load of stage s+2, two
    // fragment reads for the next group / window position, and four v_perm + one LDS write that
    // move one tap (weights) or one column (activations) of stage s+1 into the other LDS buffer.
    const int stages = g.Cin / KC;            // real stages per tile
    const int stages_even = (stages + 1) & ~1;  // an odd count is padded with a stage of zeros
    u4v wreg[2][8], xreg[2][8];
    f32x16 acc[4][2][2];
    int b_lds[4][HI][HI];

    auto load_one = [&](int ci0, unsigned wv, unsigned xv, int j, u4v (&wr)[8], u4v (&xr)[8]) {
        if (j < 8)
            wr[j] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, wv,
                                                          (unsigned)((ci0 + j) * (NN * 2)), 0);
        else
            xr[j - 8] = __builtin_amdgcn_raw_buffer_load_b128(
                rs_x, xv, (unsigned)(ci0 + j - 8) * x_cstride, 0);
    };
    auto store_one = [&](int buf, int j, const u4v (&wr)[8], const u4v (&xr)[8]) {
        if (j < 8)
            *reinterpret_cast<u4v*>(lds + buf * WS_STAGE + w_lds + j * W_PLANE) = transposed_row(wr, j);
        else
            *reinterpret_cast<u4v*>(lds + XS_OFF + buf * XS_STAGE_MAX + x_lds + (j - 8) * 16) =
                transposed_row(xr, j - 8);
    };
    auto a_frag = [&](int buf, int p, int c) {
        const int u = p / HI, v = p % HI, r = c >> 1, sc = c & 1;
        const int tap = (r + 2 * u) * N + (sc + 2 * v);
        return *reinterpret_cast<const bf16x8*>(lds + buf * WS_STAGE + a_lds + tap * W_PLANE);
    };
    auto b_frag = [&](int buf, int p, int nt) {
        return *reinterpret_cast<const bf16x8*>(lds + b_lds[nt][p / HI][p % HI] + buf * XS_STAGE_MAX);
    };
    // one K stage; `set` is a literal at every call site so that all indices fold.  (ci_next, wv,
    // xv) describe the stage requested from memory during this one.
    auto stage = [&](int set, int ci_next, unsigned wv, unsigned xv) {
        constexpr int NG = grp_count(N);  // 16 or 9
        bf16x8 bf[2][4], af[3];
#pragma unroll
        for (int i = 0; i < 4; ++i) bf[0][i] = b_frag(set, 0, i);
        af[0] = a_frag(set, grp_at(N, 0) >> 2, grp_at(N, 0) & 3);
        af[1] = a_frag(set, grp_at(N, 1) >> 2, grp_at(N, 1) & 3);
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
            const int p = grp_at(N, gi) >> 2, c = grp_at(N, gi) & 3, rank = grp_rank(N, gi);
            // the 16 staging items of a stage (8 weight rows, 8 activation rows) are dealt to
            // the groups: one each for n = 4, one or two for n = 3
            const int it0 = gi * 16 / NG, it1 = (gi + 1) * 16 / NG;
            // A wave issues in order and waits for the matrix pipe at every MFMA, so the other
            // instructions are spread one by one into the shadows of the four MFMAs of a group:
            // global load | fragment reads (two groups ahead: LDS latency under load exceeds
            // one group) | v_perm | LDS write.
            auto mfma = [&](int nt) {
                __builtin_amdgcn_sched_barrier(0);
                acc[nt][c >> 1][c & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    af[gi % 3], bf[p & 1][nt], acc[nt][c >> 1][c & 1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            };
            auto item_row = [&](int it) {
                return it < 8 ? transposed_row(wreg[set ^ 1], it) : transposed_row(xreg[set ^ 1], it - 8);
            };
            auto item_write = [&](int it, const u4v& t) {
                if (it < 8)
                    *reinterpret_cast<u4v*>(lds + (set ^ 1) * WS_STAGE + w_lds + it * W_PLANE) = t;
                else
                    *reinterpret_cast<u4v*>(lds + XS_OFF + (set ^ 1) * XS_STAGE_MAX + x_lds + (it - 8) * 16) = t;
            };
            mfma(0);
            load_one(ci_next, wv, xv, it0, wreg[set], xreg[set]);
            mfma(1);
            if (gi + 2 < NG) af[(gi + 2) % 3] = a_frag(set, grp_at(N, gi + 2) >> 2, grp_at(N, gi + 2) & 3);
            // the first two groups of a window position fetch the next position's fragments
            if (p + 1 < HI * HI && rank < 2) {
                bf[(p + 1) & 1][2 * rank] = b_frag(set, p + 1, 2 * rank);
                bf[(p + 1) & 1][2 * rank + 1] = b_frag(set, p + 1, 2 * rank + 1);
            }
            if (it1 - it0 > 1) load_one(ci_next, wv, xv, it0 + 1, wreg[set], xreg[set]);
            mfma(2);
            const u4v t0 = item_row(it0);
            u4v t1 = t0;
            if (it1 - it0 > 1) t1 = item_row(it0 + 1);
            mfma(3);
            item_write(it0, t0);
            if (it1 - it0 > 1) item_write(it0 + 1, t1);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- first tile of this block: fill the pipeline
    int cb = 0, qt = 0;
    bool have = tile_of(0, cb, qt);
    unsigned wv_c = kInvalid, xv_c = kInvalid;
    if (have) staging_offsets(cb, qt, wv_c, xv_c);
#pragma unroll
    for (int j = 0; j < 16; ++j) load_one(0, wv_c, xv_c, j, wreg[0], xreg[0]);
    {
        const bool real = stages > 1;
#pragma unroll
        for (int j = 0; j < 16; ++j)
            load_one(real ? KC : 0, real ? wv_c : kInvalid, real ? xv_c : kInvalid, j, wreg[1], xreg[1]);
    }
    __syncthreads();  // zero fill done before the first activation writes
#pragma unroll
    for (int j = 0; j < 16; ++j) store_one(0, j, wreg[0], xreg[0]);
    __syncthreads();

    for (int rho = 0; have; ++rho) {
        // next tile of this block (its first two stages are fetched during this tile's last two)
        int cb_n = 0, qt_n = 0;
        const bool have_n = tile_of(rho + 1, cb_n, qt_n);
        unsigned wv_n = kInvalid, xv_n = kInvalid;
        if (have_n) staging_offsets(cb_n, qt_n, wv_n, xv_n);

        // B (activations): lane = quad q0 + qh*128 + nt*32 + l32 of this tile, k-half gk
        const int q0 = qt * TN;
        const int q_last = (q0 + TN - 1 < a.Q ? q0 + TN - 1 : a.Q - 1);
        const int bf0 = fdiv(q0, a.dKHW), kf0 = fdiv(q0 - bf0 * KHW, a.dKW);
        const int e_first = bf0 * a.EH + kf0;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            int q = q0 + qh * 128 + nt * 32 + l32;
            if (q >= a.Q) q = q_last;
            const int b = fdiv(q, a.dKHW);
            const int rem = q - b * KHW;
            const int kk = fdiv(rem, a.dKW), mm = rem - kk * g.KW;
            const int r = b * a.EH + kk - e_first;
#pragma unroll
            for (int u = 0; u < HI; ++u)
#pragma unroll
                for (int v = 0; v < HI; ++v) {
                    const int c = mm + v + (a.OFFS - (g.P >> 1));  // LDS column of window column v
                    b_lds[nt][u][v] = XS_OFF + ((gk * a.ROWS + r + u) * a.LWS + c + (c >> 3)) * 16;
                }
        }
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int sc = 0; sc < 2; ++sc)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[nt][r][sc][i] = 0.f;

        // In iteration s the loads of stage s+2 go into register set 0 and those of s+3 into set 1
        // (their previous contents are already in LDS), while sets 1 / 0 are transposed into the
        // other LDS buffer.  The last iteration requests stages 0 and 1 of the next tile instead.
        for (int s = 0; s < stages_even; s += 2) {
            const bool last = s + 2 >= stages_even;
            {
                const int t = last ? 0 : s + 2;
                stage(0, t * KC, last ? wv_n : wv_c, last ? xv_n : xv_c);
            }
            __syncthreads();
            {
                const int t = last ? 1 : s + 3;
                const bool real = t < stages;
                stage(1, real ? t * KC : 0, real ? (last ? wv_n : wv_c) : kInvalid,
                      real ? (last ? xv_n : xv_c) : kInvalid);
            }
            __syncthreads();
        }

        // ---- drain: accumulator register i of a tile holds channel 8*(i/4) + 4*gk + (i%4) of the
        // wave's 32, for the lane's quad; column classes s = 1, 0 are neighbours in memory
        const int co0 = cb * TM;
        unsigned off_pair[4][2], off_s1[4][2], off_s0[4][2];
        bool any_edge[4][2];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            const int q = q0 + qh * 128 + nt * 32 + l32;
            const bool qv = q < a.Q;
            const int qq = qv ? q : q_last;
            const int b = fdiv(qq, a.dKHW);
            const int rem = qq - b * KHW;
            const int kk = fdiv(rem, a.dKW), mm = rem - kk * g.KW;
            const int k = g.k_min + kk, m = g.m_min + mm;
            const int oy1 = 2 * k - 1 - g.P, ox1 = 2 * m - 1 - g.P;  // row / column of class 1
            const bool vcol1 = ox1 >= 0 && ox1 < g.OW, vcol0 = ox1 + 1 < g.OW;
            const unsigned y_off =
                (unsigned)(((b * g.Cout + co0 + cw * 32 + 4 * gk) * g.OH + oy1) * g.OW + ox1) * ES;
#pragma unroll
            for (int r = 1; r >= 0; --r) {
                const bool vrow = qv && (r ? (oy1 >= 0 && oy1 < g.OH) : (oy1 + 1 < g.OH));
                const unsigned base = y_off + (r ? 0u : (unsigned)g.OW * ES);
                off_pair[nt][r] = (vrow && vcol1 && vcol0) ? base : kInvalid;
                off_s1[nt][r] = (vrow && vcol1 && !vcol0) ? base : kInvalid;
                off_s0[nt][r] = (vrow && !vcol1 && vcol0) ? base + ES : kInvalid;
                const bool edge = (off_s1[nt][r] != kInvalid) || (off_s0[nt][r] != kInvalid);
                any_edge[nt][r] = __builtin_amdgcn_ballot_w64(edge) != 0;  // wave-uniform
            }
        }
        // channel outermost, quad tiles innermost: the four stores of an inner loop write one
        // contiguous run of an output row
        auto drain = [&](auto act_tag) {
            constexpr int ACT = decltype(act_tag)::value;  // -1: no epilogue at all
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                // (a partial last channel block: groups of 8 channels exist or not as a whole)
                if (co0 + cw * 32 + 8 * (i / 4) >= g.Cout) continue;
                const unsigned soff = (unsigned)(8 * (i / 4) + (i % 4)) * plane;
                float bv = 0.f;
                if constexpr (ACT >= 0)
                    if (ep.bias) {
                        // both candidates through wave-uniform indices of a constant-address-space
                        // view (the bias is never written here): scalar loads, which do not queue
                        // behind the drain's stores the way a per-lane vector load would
                        const int ch = co0 + cw * 32 + 8 * (i / 4) + (i % 4);
                        const bias_cptr bp = (bias_cptr)(unsigned long long)ep.bias;
                        const float b_lo = bp[ch], b_hi = bp[ch + 4];
                        bv = gk ? b_hi : b_lo;
                    }
#pragma unroll
                for (int r = 1; r >= 0; --r)
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) {
                        u2v d;
                        float v1 = acc[nt][r][1][i], v0 = acc[nt][r][0][i];  // by value, then bits
                        if constexpr (ACT >= 0) {
                            v1 = epilogue_t<ACT>(v1, bv);
                            v0 = epilogue_t<ACT>(v0, bv);
                        }
                        if constexpr (OUT16) {
                            // column ox1 (class s = 1) in the low half: the lower address
                            const bf16x2 pk = {(__bf16)v1, (__bf16)v0};
                            const unsigned bits = __builtin_bit_cast(unsigned, pk);
                            __builtin_amdgcn_raw_buffer_store_b32(bits, rs_y, off_pair[nt][r], soff, 0);
                            if (any_edge[nt][r]) {
                                __builtin_amdgcn_raw_buffer_store_b16((short)(bits & 0xFFFFu), rs_y,
                                                                      off_s1[nt][r], soff, 0);
                                __builtin_amdgcn_raw_buffer_store_b16((short)(bits >> 16), rs_y,
                                                                      off_s0[nt][r], soff, 0);
                            }
                        } else {
                            d.x = __float_as_uint(v1);
                            d.y = __float_as_uint(v0);
                            __builtin_amdgcn_raw_buffer_store_b64(d, rs_y, off_pair[nt][r], soff, 0);
                            if (any_edge[nt][r]) {
                                __builtin_amdgcn_raw_buffer_store_b32(d.x, rs_y, off_s1[nt][r], soff, 0);
                                __builtin_amdgcn_raw_buffer_store_b32(d.y, rs_y, off_s0[nt][r], soff, 0);
                            }
                        }
                    }
            }
        };
        if constexpr (EPI) with_activation(ep.act, drain);  // one uniform branch per tile
        else drain(std::integral_constant<int, -1>{});
        have = have_n; cb = cb_n; qt = qt_n; wv_c = wv_n; xv_c = xv_n;
    }
}

bool make_args(const Geom& g, int dtype, MfmaArgs& a)
{
    if (dtype != 1 && dtype != 2) return false;  // fp32 operands: see ukst_mfma_f32.hip
    if (g.n != 4 && g.n != 3) return false;
    // (whole groups of 8 output channels: a partial last channel block skips the missing groups)
    if (g.Cin % KC != 0 || g.Cout % 8 != 0) return false;
    if (g.W % 8 != 0) return false;              // 16-byte row chunks
    const size_t xbytes = (size_t)g.B * g.Cin * g.H * g.W * 2;
    const size_t wbytes = (size_t)g.Cout * g.Cin * g.n * g.n * 2;
    const size_t ybytes = (size_t)g.B * g.Cout * g.OH * g.OW * 4;
    const size_t lim = 0x7FFFFFF0u;              // single buffer descriptors, 32-bit byte offsets
    if (xbytes > lim || wbytes > lim || ybytes > lim) return false;
    const int HI = (g.n + 1) / 2;
    a.g = g;
    const long long Q = (long long)g.B * g.KH * g.KW;
    if (Q > 0x7FFFFFFFLL - TN) return false;
    a.Q = (int)Q;
    a.EH = g.KH + HI - 1;
    // 256 consecutive flattened quads touch at most this many quad rows / images
    const int nrho = (TN - 2) / g.KW + 2;
    const int nimg = (TN - 2) / (g.KH * g.KW) + 2;
    a.ROWS = nrho + (HI - 1) * nimg;
    a.OFFS = ((g.P >> 1) + 7) & ~7;
    int LW = a.OFFS + g.W + HI;  // columns: left halo, the row, right halo
    const int need = g.KW + HI - 1 + (a.OFFS - (g.P >> 1));
    if (LW < need) LW = need;
    a.LWS = LW + (LW >> 3) + 1;
    a.C8 = g.W / 8;
    if (2 * a.ROWS * a.LWS * 16 > XS_STAGE_MAX) return false;
    if (a.ROWS * 2 * a.C8 > 256) return false;   // one staging unit per thread
    a.nco = (g.Cout + TM - 1) / TM;
    a.nqt = (int)((Q + TN - 1) / TN);
    if ((long long)a.nco * a.nqt > 0x3FFFFFFFLL) return false;
    a.ntiles = a.nco * a.nqt;
    // keep in one L2 what is bigger: the weights of a channel block or a tile's activations
    a.cb_major = ((size_t)TM * g.Cin * g.n * g.n * 2 > (size_t)(1 << 20)) ? 1 : 0;
    a.dKHW = make_fastdiv((unsigned)(g.KH * g.KW));
    a.dKW = make_fastdiv((unsigned)g.KW);
    a.dEH = make_fastdiv((unsigned)a.EH);
    a.dC8 = make_fastdiv((unsigned)a.C8);
    a.dROWS = make_fastdiv((unsigned)a.ROWS);
    a.dNCO = make_fastdiv((unsigned)a.nco);
    a.dNQT = make_fastdiv((unsigned)a.nqt);
    return true;
}

}  // namespace

// The output-aligned kernel runs every layer it takes (even P): no edge quads, 16-byte drain
// stores.  Measured against the shifted quads of this file: 128x128 maps 557 vs 584 us, 16x16 maps
// (289 vs 256 quads per image) 227 vs 279 us.  The shifted quads keep odd P, where they ARE the
// aligned ones.
static bool prefer_aligned(const Geom& g, int dtype)
{
    return mfma_aligned_supported(g, dtype);
}

// true if a bf16 layer runs on the bf16 matrix pipe (else, if at all, on the fp32 pipe with
// widened operands: kernel sides other than 4)
static bool bf16_pipe(const Geom& g, int dtype)
{
    MfmaArgs a;
    return dtype != 0 && (mfma_aligned_supported(g, dtype) || make_args(g, dtype, a));
}

bool mfma_supported(const Geom& g, int dtype)
{
    if (dtype == 0) return mfma_f32_supported(g, dtype) || thin_mfma_supported(g, dtype);
    MfmaArgs a;
    return mfma_aligned_supported(g, dtype) || make_args(g, dtype, a) || mfma_f32_supported(g, dtype);
}

bool mfma_needs_aligned_x(const Geom& g, int dtype)
{
    if (dtype != 0) return bf16_pipe(g, dtype);  // the bf16 kernels move x in 16-byte pieces
    return !mfma_f32_supported(g, dtype) && thin_mfma_supported(g, dtype);
}

hipError_t launch_mfma(const Geom& g, const void* x, const void* w, float* y, int dtype,
                       Workspace& ws, hipStream_t stream)
{
    if (mfma_f32_supported(g, dtype) && (dtype == 0 || !bf16_pipe(g, dtype)))
        return launch_mfma_f32(g, x, w, y, dtype, ws, stream);
    if (ws.query) return hipSuccess;  // the kernels below use no scratch
    if (dtype == 0) return launch_thin_mfma(g, x, w, y, stream);
    if (prefer_aligned(g, dtype)) return launch_mfma_aligned(g, x, w, y, dtype, stream);
    MfmaArgs a;
    if (!make_args(g, dtype, a)) return hipErrorInvalidValue;
    const size_t lds = 2 * (size_t)(2 * W_HALF) + 2 * (size_t)XS_STAGE_MAX;
    // more than 64 KiB of dynamic LDS has to be allowed per device (a property of the loaded
    // kernel, not library state); cheap enough to repeat on every call
    const bool epi = has_epilogue(g.ep), out16 = dtype == 2;
    typedef void (*kernel_t)(const uint16_t*, const uint16_t*, void*, MfmaArgs, Epilogue);
    const kernel_t k4 = out16 ? (epi ? ukst_mfma_bf16_kernel<4, true, true> : ukst_mfma_bf16_kernel<4, false, true>)
                              : (epi ? ukst_mfma_bf16_kernel<4, true, false> : ukst_mfma_bf16_kernel<4, false, false>);
    const kernel_t k3 = out16 ? (epi ? ukst_mfma_bf16_kernel<3, true, true> : ukst_mfma_bf16_kernel<3, false, true>)
                              : (epi ? ukst_mfma_bf16_kernel<3, true, false> : ukst_mfma_bf16_kernel<3, false, false>);
    const kernel_t kfn = g.n == 3 ? k3 : k4;
    hipError_t e = hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    // persistent blocks: one per compute unit (a multiple of the 8 XCDs), never more than tiles
    int dev = 0, cus = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess)
        return e;
    int grid = (cus / 8) * 8;
    if (grid < 8) grid = 8;
    const int need = ((a.ntiles + 7) / 8) * 8;
    if (grid > need) grid = need;
    // The slowest block walks ceil(tiles / grid) tiles whatever the rest do: use only as many
    // blocks as that round count needs (584 tiles take 3 rounds on 256 blocks and on 200), the
    // idle compute units leave power for the clock of the busy ones.
    {
        const int rounds = (a.ntiles + grid - 1) / grid;
        const int fewer = (((a.ntiles + rounds - 1) / rounds + 7) / 8) * 8;
        if (fewer < grid) grid = fewer;
    }
    hipLaunchKernelGGL(kfn, dim3((unsigned)grid), dim3(256), lds, stream, (const uint16_t*)x,
                       (const uint16_t*)w, (void*)y, a, g.ep);
    return hipGetLastError();
}

const char* mfma_kernel_name(const Geom& g, int dtype)
{
    if (bf16_pipe(g, dtype))  // bf16 in; fp32 or bf16 out
        return prefer_aligned(g, dtype) ? "ukst_mfma_bf16_aligned_kernel" : "ukst_mfma_bf16_kernel";
    return mfma_f32_supported(g, dtype) ? "ukst_mfma_f32_kernel" : "ukst_thin_mfma_kernel";
}

}  // namespace ukst
