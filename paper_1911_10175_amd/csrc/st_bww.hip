// Filter-gradient kernels (BWW), unit stride: zero-skipping (vector ALUs) and dense (matrix cores).
//
// Mapping of SparseTrain Sec. 3.4 (Alg. 4-5) onto a CDNA wavefront:
//  * The filter-gradient accumulators are stationary (Sec. 3.4: T gradient vectors stay in
//    registers for the whole sweep): a wavefront owns 64 output channels (one per lane) times
//    8 input channels times R*S taps = 72 registers per lane for a 3x3 filter, which leaves room
//    for 4 wavefronts per SIMD; the scalar work of the zero tests of one wavefront then overlaps
//    the vector work of the others.
//  * The tested operand is the input x.  The tile of x for 64 input channels is staged in LDS by
//    the workgroup (8 wavefronts = 4 channel blocks x 2 halves); with unit stride both tiles are
//    double-buffered and filled by loads that write LDS directly, one tile ahead.  For four pixels at a time one
//    LDS read with a lane per (pixel, channel) followed by one compare and a ballot gives the
//    non-zero mask (the vector compare of Alg. 5, along channels and pixels instead of along the
//    minibatch: the accumulators do not depend on the pixel, so no minibatch transposition of
//    the layout is needed).  Each set bit costs one scalar bit test and branch; the value itself
//    reaches all lanes through a same-address (broadcast) LDS read of the pixel's 8 channels.
//    Which 8 of the 64 channels a wavefront takes is decided per workgroup: the channels with a non-zero in
//    the first tile of its range are dealt round the wavefronts first (whole dead planes would otherwise
//    leave some wavefronts idle at the barrier of every tile).
//  * The other operand, dy at the R*S neighbouring output pixels, is a vector over the lane's
//    output channel read from the LDS halo tile; the 3x6 window of four adjacent pixels is read
//    once per group.
//  * The sum over the minibatch and the image is split over workgroups; each writes a partial
//    gradient to the workspace and a second kernel adds the partials in a fixed order
//    (Sec. 3.4, accumulation of partial results at the end of a sweep), so results are
//    deterministic without floating-point atomics.
#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "st_common.hpp"

namespace st {
namespace {

struct BwwArgs {
    int N, C, K, H, W, OH, OW, pw, ph;
    int tiles_w, tiles_h;      // tiles over the input image (sparse) / the output image (dense)
    int units;                 // N * tiles_h * tiles_w
    int splits;                // partial sums; gridDim.x
    int cgroups;               // ceil(C/64)
    // operand selection on the device (st_conv_bww_auto): when sel is set, the launch does nothing
    // unless the sampled zero counts pick the form this launch computes (want: 0 = tests x, 1 = tests dy,
    // 2 = dense; kEitherOperand: a zero-skipping launch that carries the arguments of both of its forms
    // and computes the one selected)
    const unsigned *sel;
    int want;
    // the caller exchanged the operands (dy is the tested one): the tested channels are then the
    // layer's output channels, the lanes its input channels, and the taps come out reversed; the
    // partial sums are still written in the layer's own filter layout
    int swapped;
};

constexpr int kEitherOperand = -1;

// Which of the two argument sets a zero-skipping launch works with.  Returns false when this workgroup
// has nothing to do: the form it computes was not selected, or it lies outside the selected form's grid.
__device__ __forceinline__ bool bww_pick(BwwArgs &A, const BwwArgs &B, const float *&tested, const float *&other)
{
    if (!A.sel) return true;
    const int f = selected_form(A.sel);
    if (A.want != kEitherOperand) return f == A.want;
    if (f == 2) return false;
    if (f == 1) {
        A = B;
        const float *t = tested; tested = other; other = t;
    }
    return (int)blockIdx.x < A.splits && (int)blockIdx.y < ((A.K + 63) / 64) * A.cgroups;
}


// PSTEP = stride of the layer (1 or 2): positions of the halo between neighbouring tile pixels
template <int R, int S, int TH, int TW, int PSTEP = 1>
struct BwwCfg {
    static constexpr int HH = (TH - 1) * PSTEP + S, HW = (TW - 1) * PSTEP + R, HP = HH * HW;
};

// How the pixels of the tested tile, the taps and the pixels of the other operand's halo relate in
// the zero-skipping kernel.  A group is GP = 4 consecutive tested pixels of row a starting at
// column b0; its multiply-adds read a window of the halo that is loaded into registers once.
//   MODE 0  unit stride: pixel j, tap (v,u) <-> window [S-1-v][j+R-1-u]  (window S x (GP+R-1) at (a, b0))
//   MODE 1  stride 2, padding 1, x tested: x pixel (a, b0+j) meets dy row (a+1-v)/2 for the v that make
//           this an integer, the same along the width (window 2 x 3 at (a/2, b0/2); 1, 2 or 4 taps)
//   MODE 2  stride 2, dy tested (operands exchanged by the caller): dy pixel (a, b0+j) meets x pixel
//           (2a+v, 2(b0+j)+u) of its halo for all taps (window 3 x 9 at (2a, 2*b0)); the partial sums
//           are stored with the taps reversed, which is what the exchanged-roles reduction expects
template <int R, int S, int TH, int TW, int MODE>
struct BwwSparseCfg {
    static constexpr int GP = 4;
    static constexpr int HH = MODE == 0 ? TH + S - 1 : MODE == 1 ? TH / 2 + 1 : 2 * (TH - 1) + S;
    static constexpr int HW = MODE == 0 ? TW + R - 1 : MODE == 1 ? TW / 2 + 1 : 2 * (TW - 1) + R;
    static constexpr int HP = HH * HW;
    static constexpr int WR = MODE == 1 ? 2 : S;
    static constexpr int WC = MODE == 0 ? GP + R - 1 : MODE == 1 ? GP / 2 + 1 : 2 * (GP - 1) + R;
    static constexpr int RU = MODE == 1 ? 2 : 1;            // rows whose code differs (row parity)
    static constexpr int wrow0(int a) { return MODE == 0 ? a : MODE == 1 ? a / 2 : 2 * a; }
    static constexpr int wcol0(int b0) { return MODE == 0 ? b0 : MODE == 1 ? b0 / 2 : 2 * b0; }
    static constexpr bool valid(int par, int j, int v, int u)
    {
        return MODE != 1 || (((par + 1 - v) % 2 == 0) && ((j + 1 - u) % 2 == 0));
    }
    static constexpr int wr(int par, int v) { return MODE == 0 ? S - 1 - v : MODE == 1 ? (par + 1 - v) / 2 : v; }
    static constexpr int wc(int j, int u) { return MODE == 0 ? j + R - 1 - u : MODE == 1 ? (j + 1 - u) / 2 : 2 * j + u; }
    static constexpr int slot(int v, int u) { return MODE == 2 ? (S - 1 - v) * R + (R - 1 - u) : v * R + u; }
};

// ------------------------------------------------------------------------------------------
// zero-skipping kernel: tiles run over the INPUT image; LDS holds the x tile (64 channels) and
// the dy halo of the tile (64 output channels)
// ------------------------------------------------------------------------------------------
// x = the tested operand, dy = the other one (the caller exchanges them for the forms that test dy).
// ASYNC (unit stride): both tiles are double-buffered in dynamic LDS (bww_async_lds_bytes) and filled by loads
// that write LDS directly, no registers in between: the tile after the current one is requested right after
// the barrier that opens the current tile's work and lands during it, so no memory round trip is waited for
// and a tile costs one barrier instead of two.
typedef const __attribute__((address_space(1))) void *GlobalPtr;
typedef __attribute__((address_space(3))) void *LdsPtr;
static __device__ __attribute__((aligned(16))) float kZeros16[4] = {0.f, 0.f, 0.f, 0.f};     // source of padding
template <int R, int S, int TH, int TW>
constexpr size_t bww_async_lds_bytes()
{
    using Cfg = BwwSparseCfg<R, S, TH, TW, 0>;
    return (size_t)2 * (Cfg::HP + TH * TW) * 64 * sizeof(float);
}

template <int R, int S, int TH, int TW, int MODE, bool ASYNC = false>
__device__ __forceinline__ void bww_sparse_body(const BwwArgs &A, const float *__restrict__ x, const float *__restrict__ dy,
                                                float *__restrict__ part)
{
    using Cfg = BwwSparseCfg<R, S, TH, TW, MODE>;
    constexpr int HW = Cfg::HW, HP = Cfg::HP, TP = TH * TW;
    constexpr int CH = 8;                 // input channels per wavefront
    constexpr int GP = Cfg::GP;           // pixels per group
    static_assert(TW % GP == 0, "groups must not straddle rows");
    static_assert(TH % Cfg::RU == 0, "row parities come in pairs");
    static_assert(!ASYNC || MODE == 0, "the double-buffered form exists for unit stride only");
    constexpr int WR = Cfg::WR, WC = Cfg::WC;        // dy window of a group
    __shared__ __attribute__((aligned(16))) float dyT_static[ASYNC ? 4 : HP * 64];
    __shared__ __attribute__((aligned(16))) float xT_static[ASYNC ? 4 : TP * 64];
    extern __shared__ __attribute__((aligned(16))) float bww_dynamic_lds[];      // ASYNC: [2][HP + TP][64]
    const float *dyT = dyT_static, *xT = xT_static;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int lane = threadIdx.x % kWave;
    const int split = blockIdx.x;
    const int kt = blockIdx.y / A.cgroups, cg = blockIdx.y % A.cgroups;
    const int CB = A.C / kBlk, KB = A.K / kBlk;
    const int cbl = wave >> 1, h = wave & 1;          // channel block within the group of 64, half
    const int cb = cg * 4 + cbl;
    const int k = kt * 64 + lane;

    float acc[CH][S * R];
#pragma unroll
    for (int ci = 0; ci < CH; ++ci)
#pragma unroll
        for (int t = 0; t < S * R; ++t) acc[ci][t] = 0.f;

    const int u0 = (int)((long long)A.units * split / A.splits);
    const int u1 = (int)((long long)A.units * (split + 1) / A.splits);

    // ---- which wavefront takes which of the 64 tested channels ----
    // ReLU leaves whole (image, channel) planes dead, and a wavefront's accumulators tie it to its 8 channels
    // for the whole sweep: with the channels handed out in index order a tile takes as long as the wavefront
    // that happens to hold the most alive ones.  The channels that have a non-zero in the first tile of this
    // workgroup's range are therefore dealt round the 8 wavefronts first, the others after them: xT holds
    // channel c at position slot_of[c], and wavefront w works on positions 8w .. 8w+7 as before.  The first
    // tile is a prediction only (a channel that turns out alive later is computed like any other), and every
    // accumulator still sees its pixels in the same order: the results do not depend on the assignment.
    // With exchanged operands the order stays as it is (the 16-byte stores of that epilogue need it).
    __shared__ unsigned alive_w[2];
    __shared__ __attribute__((aligned(16))) unsigned char slot_of[64], chan_of[64];
    if (threadIdx.x < 2) alive_w[threadIdx.x] = 0u;
    __syncthreads();
    if (!A.swapped && u0 < u1) {
        int t = u0;
        const int tw = t % A.tiles_w; t /= A.tiles_w;
        const int th = t % A.tiles_h;
        const int n = t / A.tiles_h;
        unsigned nib = 0u;                                   // a thread's slots all have the same channel quarter
        for (int idx = threadIdx.x; idx < TP * 16; idx += 512) {
            const int pix = idx >> 4, q = idx & 15;
            const int ih = th * TH + pix / TW, iw = tw * TW + pix % TW;
            const int cbq = cg * 4 + (q >> 2);
            if (ih < A.H && iw < A.W && cbq < CB) {
                const float4 val = *reinterpret_cast<const float4 *>(x + act_off(n, cbq, ih, iw, CB, A.H, A.W) + (q & 3) * 4);
                nib |= (val.x != 0.f ? 1u : 0u) | (val.y != 0.f ? 2u : 0u) | (val.z != 0.f ? 4u : 0u) | (val.w != 0.f ? 8u : 0u);
            }
        }
        const int q = threadIdx.x & 15;
        if (nib) atomicOr(&alive_w[q >> 3], nib << ((q & 7) * 4));
    }
    __syncthreads();
    // Loads that write LDS directly put a lane's piece at lane * size: channels in index order, or one 4-byte
    // piece per lane (measured: four times the load instructions cost 5 % of the kernel's time).  The
    // double-buffered form therefore keeps the index order unless at least 8 of the group's channels look dead;
    // then the workgroup stages through registers like the other forms, which can put a value anywhere for free.
    bool dealt = !A.swapped;
    {
        const unsigned long long m = ((unsigned long long)alive_w[1] << 32) | alive_w[0];
        if constexpr (ASYNC) {
            const int real = A.C - cg * 64 < 64 ? A.C - cg * 64 : 64;
            const unsigned long long realmask = real == 64 ? ~0ull : (1ull << real) - 1ull;
            dealt = dealt && __builtin_popcountll(~m & realmask) >= 8;
        }
        if (threadIdx.x < 64) {
            const int c = threadIdx.x;
            const unsigned long long below = (1ull << c) - 1ull;
            const int s = (m >> c) & 1ull ? __builtin_popcountll(m & below)
                                          : __builtin_popcountll(m) + __builtin_popcountll(~m & below);
            const int slot = dealt ? (s & 7) * 8 + (s >> 3) : c;
            slot_of[c] = (unsigned char)slot;
            chan_of[slot] = (unsigned char)c;
        }
    }
    // (the barrier at the top of the tile loop orders these writes before their first use)
    const bool wave_active = A.swapped ? cb < CB : true;

    // ASYNC, channels in index order: request tile `unit` into buffer b, 16 bytes per lane: a wavefront's 64 pieces
    // are 4 pixels of [pixel][64 channels].  Lanes outside the image or beyond the channel count read zeros
    // from kZeros16; lanes beyond the buffer are switched off.  The LDS address of an instruction is the same in
    // every lane (the hardware adds lane * size).
    auto issue = [&](int unit, int b) __attribute__((always_inline)) {
        int t = unit;
        const int tw = t % A.tiles_w; t /= A.tiles_w;
        const int th = t % A.tiles_h;
        const int n = t / A.tiles_h;
        const int ih0 = th * TH, iw0 = tw * TW;
        const int ohs = ih0 + A.ph - (S - 1), ows = iw0 + A.pw - (R - 1);
        float *dst_dy = bww_dynamic_lds + b * ((HP + TP) * 64), *dst_x = dst_dy + HP * 64;
        int ln = lane;
        asm volatile("" : "+v"(ln));                     // (addresses recomputed per tile, not kept in registers)
        constexpr int NI = (HP * 16 + 63) / 64;
        for (int i = wave; i < NI; i += 8) {
            const int idx = i * 64 + ln;
            const int pix = idx >> 4, q = idx & 15;
            const int oh = ohs + pix / HW, ow = ows + pix % HW;
            const int kb = kt * 4 + (q >> 2);
            const float *src = kZeros16;
            if (idx < HP * 16 && oh >= 0 && oh < A.OH && ow >= 0 && ow < A.OW && kb < KB)
                src = dy + act_off(n, kb, oh, ow, KB, A.OH, A.OW) + (q & 3) * 4;
            if (idx < HP * 16)
                __builtin_amdgcn_global_load_lds((GlobalPtr)src, (LdsPtr)(dst_dy + i * 256), 16, 0, 0);
        }
        constexpr int NIX = TP * 16 / 64;
        for (int i = wave; i < NIX; i += 8) {
            const int idx = i * 64 + ln;
            const int pix = idx >> 4, q = idx & 15;
            const int ih = ih0 + pix / TW, iw = iw0 + pix % TW;
            const int cbq = cg * 4 + (q >> 2);
            const float *src = kZeros16;
            if (ih < A.H && iw < A.W && cbq < CB) src = x + act_off(n, cbq, ih, iw, CB, A.H, A.W) + (q & 3) * 4;
            __builtin_amdgcn_global_load_lds((GlobalPtr)src, (LdsPtr)(dst_x + i * 256), 16, 0, 0);
        }
    };
    if constexpr (ASYNC) {
        __syncthreads();                                 // the tables are written
        if (u0 < u1 && !dealt) issue(u0, 0);
    }

    // lane -> (pixel of the group, channel of the block) for the mask read
    const int mpix = lane >> 4, mch = lane & 15;

    for (int unit = u0; unit < u1; ++unit) {
        int t = unit;
        const int tw = t % A.tiles_w; t /= A.tiles_w;
        const int th = t % A.tiles_h;
        const int n = t / A.tiles_h;
        const int ih0 = th * TH, iw0 = tw * TW;
        // first halo pixel of the other operand (MODE 1 assumes padding 1 and even tile origins)
        const int ohs = MODE == 0 ? ih0 + A.ph - (S - 1) : MODE == 1 ? ih0 / 2 : 2 * ih0 - A.ph;
        const int ows = MODE == 0 ? iw0 + A.pw - (R - 1) : MODE == 1 ? iw0 / 2 : 2 * iw0 - A.pw;

        if (ASYNC && !dealt) {
            const int b = (unit - u0) & 1;
            __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): this wavefront's pieces of the tile have landed
            __syncthreads();                                 // everyone's have; everyone is done with the previous tile
            dyT = bww_dynamic_lds + b * ((HP + TP) * 64);
            xT = dyT + HP * 64;
            if (unit + 1 < u1) issue(unit + 1, b ^ 1);       // lands during this tile's work
        } else {
            // dy[n, kt*64 .. +63, halo] as [pixel][64 k]; x[n, cg*64 .. +63, tile] as [pixel][64 c];
            // 16 float4 per pixel, zeros outside the image and beyond the channel count.  A thread asks for all its
            // 16-byte pieces of the next tile at once, and before the barrier: their round trip overlaps the wait
            // for the wavefronts still at work on the previous tile (one load, one wait, one LDS write at a time,
            // which is what the plain loop compiles to, makes six round trips per tile).
            float *sdst_dy = ASYNC ? bww_dynamic_lds : dyT_static, *sdst_x = ASYNC ? bww_dynamic_lds + HP * 64 : xT_static;
            if constexpr (ASYNC) {
                dyT = sdst_dy;
                xT = sdst_x;
            }
            constexpr int NDY = (HP * 16 + 511) / 512, NX = (TP * 16 + 511) / 512;
            float4 sdy[NDY], sx[NX];
            // (the slot arithmetic is redone for every tile from a thread index the compiler cannot see through:
            // kept across the tile's work as address registers, it spills)
            int tid = threadIdx.x;
            asm volatile("" : "+v"(tid));
#pragma unroll
            for (int i = 0; i < NDY; ++i) {
                const int idx = tid + i * 512;
                const int pix = idx >> 4, q = idx & 15;
                const int oh = ohs + pix / HW, ow = ows + pix % HW;
                const int kb = kt * 4 + (q >> 2);
                sdy[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (idx < HP * 16 && oh >= 0 && oh < A.OH && ow >= 0 && ow < A.OW && kb < KB)
                    sdy[i] = *reinterpret_cast<const float4 *>(dy + act_off(n, kb, oh, ow, KB, A.OH, A.OW) + (q & 3) * 4);
            }
#pragma unroll
            for (int i = 0; i < NX; ++i) {
                const int idx = tid + i * 512;
                const int pix = idx >> 4, q = idx & 15;
                const int ih = ih0 + pix / TW, iw = iw0 + pix % TW;
                const int cbq = cg * 4 + (q >> 2);
                sx[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (idx < TP * 16 && ih < A.H && iw < A.W && cbq < CB)
                    sx[i] = *reinterpret_cast<const float4 *>(x + act_off(n, cbq, ih, iw, CB, A.H, A.W) + (q & 3) * 4);
            }
            __syncthreads();                                     // every wavefront is done with the previous tile
#pragma unroll
            for (int i = 0; i < NDY; ++i) {
                const int idx = tid + i * 512;
                if (idx < HP * 16) *reinterpret_cast<float4 *>(sdst_dy + idx * 4) = sdy[i];       // = [pix][q*4]
            }
            {
                const unsigned sl = reinterpret_cast<const unsigned *>(slot_of)[tid & 15];     // positions of channels 4q .. 4q+3
#pragma unroll
                for (int i = 0; i < NX; ++i) {
                    const int idx = tid + i * 512;
                    const int pix = idx >> 4;
                    if (idx < TP * 16) {
                        sdst_x[pix * 64 + (sl & 0xffu)] = sx[i].x;
                        sdst_x[pix * 64 + ((sl >> 8) & 0xffu)] = sx[i].y;
                        sdst_x[pix * 64 + ((sl >> 16) & 0xffu)] = sx[i].z;
                        sdst_x[pix * 64 + (sl >> 24)] = sx[i].w;
                    }
                }
            }
            __syncthreads();
        }
        if (!wave_active) continue;

        // A multiply-add whose accumulator and two factors all sit in even-numbered or all in odd-numbered
        // registers issues at half rate.  The 8 tested values of a pixel arrive in two aligned groups of four
        // registers, channel ci in one of parity ci % 2; the accumulators of channels 2i + 1 and 2i are handed to
        // the register allocator as (even, odd) pairs here, so that an accumulator never has the parity of
        // its channel's tested value, wherever the window value sits.
        typedef float f2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int ci = 0; ci < CH; ci += 2)
#pragma unroll
            for (int tp = 0; tp < S * R; ++tp) {
                f2 pr = {acc[ci + 1][tp], acc[ci][tp]};
                asm volatile("" : "+v"(pr));
                acc[ci + 1][tp] = pr.x;
                acc[ci][tp] = pr.y;
            }

        // the mask values of a group are read one group ahead (groups follow each other in memory)
        float mnext = xT[mpix * 64 + cbl * 16 + mch];
        for (int rp = 0; rp < TH / Cfg::RU; ++rp)
        static_for<0, Cfg::RU>([&](auto PAR) __attribute__((always_inline)) {
        constexpr int par = decltype(PAR)::value;            // row parity (MODE 1), else 0
        const int a = rp * Cfg::RU + par;
        for (int b0 = 0; b0 < TW; b0 += GP) {                // groups of GP pixels along the row
            const int g0 = a * TW + b0;
            // non-zero mask of the group: bit 16*j + c for pixel j, channel c of the block
            const float mval = mnext;
            if (g0 + GP < TP) mnext = xT[(g0 + GP + mpix) * 64 + cbl * 16 + mch];
            const unsigned long long m64 = __builtin_amdgcn_ballot_w64(mval != 0.f);
            const unsigned mlo = (unsigned)m64, mhi = (unsigned)(m64 >> 32);
            const unsigned wlo = mlo >> (h * CH), whi = mhi >> (h * CH);     // shifted once per group, not per pixel
            // this wavefront's 8 channels of pixels 0 / 1 (wlo) and 2 / 3 (whi): bits 0-7 and 16-23
            const unsigned any = (wlo | whi) & 0x00FF00FFu;
            if (any == 0u) continue;                         // nothing to do for these 4 pixels x 8 channels
            // window of the other operand's halo, this lane's channel
            float dyw[WR][WC];
            const int w0 = Cfg::wrow0(a) * HW + Cfg::wcol0(b0);
#pragma unroll
            for (int r = 0; r < WR; ++r)
#pragma unroll
                for (int cc = 0; cc < WC; ++cc) dyw[r][cc] = dyT[(w0 + r * HW + cc) * 64 + lane];
            // x of pixel 0 of the group: 8 channels, same address in all lanes
            const float4 *xq = reinterpret_cast<const float4 *>(xT + g0 * 64 + cbl * 16 + h * CH);
            float4 xlo = xq[0], xhi = xq[1];
            __builtin_amdgcn_s_waitcnt(0xC07F);              // lgkmcnt(0): window and first pixel are here
            static_for<0, GP>([&](auto J) __attribute__((always_inline)) {
                constexpr int j = decltype(J)::value;
                float4 nlo = xlo, nhi = xhi;
                if constexpr (j + 1 < GP) {                  // next pixel's values fly during this pixel's work
                    nlo = xq[(j + 1) * 16];
                    nhi = xq[(j + 1) * 16 + 1];
                }
                const float xs[CH] = {xlo.x, xlo.y, xlo.z, xlo.w, xhi.x, xhi.y, xhi.z, xhi.w};
                // this wavefront's 8 channels of pixel j sit at constant bit positions of the shifted mask words
                const unsigned mw = (j < 2) ? wlo : whi;
                constexpr int sh = (j % 2) * 16;
                if (__builtin_expect((mw & (0xFFu << sh)) != 0u, 1)) {
                    static_for<0, CH>([&](auto CI) __attribute__((always_inline)) {
                        constexpr int ci = decltype(CI)::value;
                        if (__builtin_expect((mw & (1u << (sh + ci))) != 0u, 1)) {
#pragma unroll
                            for (int v = 0; v < S; ++v)
#pragma unroll
                                for (int u = 0; u < R; ++u)
                                    if (Cfg::valid(par, j, v, u))
                                        acc[ci][Cfg::slot(v, u)] = fmaf(xs[ci], dyw[Cfg::wr(par, v)][Cfg::wc(j, u)],
                                                                        acc[ci][Cfg::slot(v, u)]);
                        }
                    });
                }
                if constexpr (j + 1 < GP) __builtin_amdgcn_s_waitcnt(0xC07F);
                xlo = nlo;
                xhi = nhi;
            });
        }
        });
    }

    if (wave_active && k < A.K) {
        const int kb = k / kBlk, ki = k % kBlk;
        float *pbase = part + (size_t)split * A.K * A.C * (S * R);
        if (!A.swapped) {
#pragma unroll
            for (int ci = 0; ci < CH; ++ci) {
                const int c = cg * 64 + chan_of[wave * CH + ci];        // the channel this accumulator row belongs to
                if (c >= A.C) continue;
                float *p = pbase + ((size_t)kb * CB + c / kBlk) * (S * R * kBlk * kBlk) + (c % kBlk) * kBlk + ki;
#pragma unroll
                for (int tp = 0; tp < S * R; ++tp) p[tp * (kBlk * kBlk)] = acc[ci][tp];
            }
        } else {
            // layer's block [cb: its output channels][kb: its input channels], element [ki][h*8 + ci]: the
            // lane's 8 tested channels are consecutive, the taps are reversed
            // The values pass through an OR with a zero the compiler cannot see, i.e. through fresh registers:
            // handed to the 16-byte stores directly, the accumulators would have to sit in aligned groups of
            // four, and that numbering makes the multiply-adds of the main loop 6 % slower (measured), for the
            // x-testing form as well since it is the same code.
            const unsigned zero = (unsigned)(A.swapped - 1);
            auto fresh = [&](float v) __attribute__((always_inline)) { return __uint_as_float(__float_as_uint(v) | zero); };
            float *p = pbase + ((size_t)cb * KB + kb) * (S * R * kBlk * kBlk) + ki * kBlk + h * CH;
#pragma unroll
            for (int tp = 0; tp < S * R; ++tp) {
                float4 *q = reinterpret_cast<float4 *>(p + (S * R - 1 - tp) * (kBlk * kBlk));
                q[0] = make_float4(fresh(acc[0][tp]), fresh(acc[1][tp]), fresh(acc[2][tp]), fresh(acc[3][tp]));
                q[1] = make_float4(fresh(acc[4][tp]), fresh(acc[5][tp]), fresh(acc[6][tp]), fresh(acc[7][tp]));
            }
        }
    }
}

template <int R, int S, int TH, int TW, int MODE = 0>
__global__ __launch_bounds__(512, 4) void bww_sparse_kernel(BwwArgs A, const float *__restrict__ x,
                                                            const float *__restrict__ dy, float *__restrict__ part)
{
    if (deselected(A.sel, A.want)) return;              // uniform over the grid, before any barrier
    bww_sparse_body<R, S, TH, TW, MODE, MODE == 0>(A, x, dy, part);
}

// st_conv_bww_auto: one launch for both zero-skipping forms of a unit-stride layer.  It carries the arguments of
// the x-testing form (A) and of the dy-testing form (B, operands exchanged) and computes the one the sampled
// counts select; a kernel of its own, so that the kernel of the direct calls keeps its code (with the choice
// inside, that one ran 6 % slower).
template <int R, int S, int TH, int TW>
__global__ __launch_bounds__(512, 4) void bww_sparse_either_kernel(BwwArgs A, BwwArgs B, const float *x, const float *dy,
                                                                   float *__restrict__ part)
{
    const float *tested = x, *other = dy;
    if (!bww_pick(A, B, tested, other)) return;         // uniform over the workgroup, before any barrier
    bww_sparse_body<R, S, TH, TW, 0, true>(A, tested, other, part);
}

// ------------------------------------------------------------------------------------------
// dense kernel: tiles run over the OUTPUT image; LDS holds the dy tile and the x halo.
// v_mfma_f32_32x32x2_f32 with rows = 32 input channels, columns = 32 output channels, reduction
// = 2 pixels per instruction; one accumulator block per filter tap.
// ------------------------------------------------------------------------------------------
template <int R, int S, int TH, int TW, int PSTEP = 1>
__global__ __launch_bounds__(256) void bww_dense_kernel(BwwArgs A, const float *__restrict__ x,
                                                        const float *__restrict__ dy,
                                                        float *__restrict__ part)
{
    using Cfg = BwwCfg<R, S, TH, TW, PSTEP>;
    if (deselected(A.sel, A.want)) return;              // uniform over the grid, before any barrier
    constexpr int HW = Cfg::HW, HP = Cfg::HP, TP = TH * TW;
    static_assert(TW % 2 == 0, "pixel pairs must not straddle rows");
    __shared__ __attribute__((aligned(16))) float dyT[TP * 64];
    __shared__ __attribute__((aligned(16))) float xT[HP * 64];

    // the wavefront index is the same in every lane: kept in a scalar register, and with it every tile coordinate
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;
    const int l32 = lane % 32, half = lane / 32;
    const int kh = wave % 2, ch = wave / 2;
    const int split = blockIdx.x;
    const int kt = blockIdx.y / A.cgroups, cg = blockIdx.y % A.cgroups;
    const int CB = A.C / kBlk, KB = A.K / kBlk;

    floatx16 acc[S * R];
#pragma unroll
    for (int t = 0; t < S * R; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    const int u0 = (int)((long long)A.units * split / A.splits);
    const int u1 = (int)((long long)A.units * (split + 1) / A.splits);

    // A thread's 16-byte pieces of a tile (dy tile, then x halo: 16 float4 per pixel, zeros outside the image
    // and beyond the channel count) are asked for while the previous tile is being multiplied and written to LDS
    // after it: the memory round trip is hidden behind the matrix work.  (A plain staging loop compiles to
    // load, wait, write per piece: 16 round trips per tile, about as long as the tile's MFMAs.)
    constexpr int ND = (TP * 16 + 255) / 256, NXH = (HP * 16 + 255) / 256;
    float4 sd[ND], sx[NXH];
    auto fetch = [&](int unit) __attribute__((always_inline)) {
        int t = unit;
        const int tw = t % A.tiles_w; t /= A.tiles_w;
        const int th = t % A.tiles_h;
        const int n = t / A.tiles_h;
        const int oh0 = th * TH, ow0 = tw * TW;
        const int ih0 = oh0 * PSTEP - A.ph, iw0 = ow0 * PSTEP - A.pw;
        // (thread index the compiler cannot see through: the slot arithmetic is redone per tile instead of
        // being kept in address registers across the tile's work)
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
#pragma unroll
        for (int i = 0; i < ND; ++i) {
            const int idx = tid + i * 256;
            const int pix = idx >> 4, q = idx & 15;
            const int oh = oh0 + pix / TW, ow = ow0 + pix % TW;
            const int kb = kt * 4 + (q >> 2);
            sd[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (idx < TP * 16 && oh < A.OH && ow < A.OW && kb < KB)
                sd[i] = *reinterpret_cast<const float4 *>(dy + act_off(n, kb, oh, ow, KB, A.OH, A.OW) + (q & 3) * 4);
        }
#pragma unroll
        for (int i = 0; i < NXH; ++i) {
            const int idx = tid + i * 256;
            const int pix = idx >> 4, q = idx & 15;
            const int ih = ih0 + pix / HW, iw = iw0 + pix % HW;
            const int cb = cg * 4 + (q >> 2);
            sx[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (idx < HP * 16 && ih >= 0 && ih < A.H && iw >= 0 && iw < A.W && cb < CB)
                sx[i] = *reinterpret_cast<const float4 *>(x + act_off(n, cb, ih, iw, CB, A.H, A.W) + (q & 3) * 4);
        }
    };
    if (u0 < u1) fetch(u0);

    for (int unit = u0; unit < u1; ++unit) {
        __syncthreads();                                     // every wavefront is done with the previous tile
        {
            int tid = threadIdx.x;
            asm volatile("" : "+v"(tid));
#pragma unroll
            for (int i = 0; i < ND; ++i) {
                const int idx = tid + i * 256;
                if (idx < TP * 16) *reinterpret_cast<float4 *>(dyT + idx * 4) = sd[i];        // = [pix][q*4]
            }
#pragma unroll
            for (int i = 0; i < NXH; ++i) {
                const int idx = tid + i * 256;
                if (idx < HP * 16) *reinterpret_cast<float4 *>(xT + idx * 4) = sx[i];
            }
        }
        __syncthreads();
        if (unit + 1 < u1) fetch(unit + 1);                  // in flight during this tile's MFMAs

        for (int pp = 0; pp < TP / 2; ++pp) {
            const int p = 2 * pp + half;
            const int a = p / TW, b = p % TW;
            const float bv = dyT[p * 64 + kh * 32 + l32];                  // B[kk = half][j = k]
#pragma unroll
            for (int v = 0; v < S; ++v)
#pragma unroll
                for (int u = 0; u < R; ++u) {
                    const float av = xT[((a * PSTEP + v) * HW + (b * PSTEP + u)) * 64 + ch * 32 + l32];   // A[i = c][kk]
                    acc[v * R + u] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[v * R + u], 0, 0, 0);
                }
        }
    }

    // D[i = c][j = k]: column = lane % 32, row = 8*(r/4) + 4*(lane/32) + r%4
    const int k = kt * 64 + kh * 32 + l32;
    if (k < A.K) {
        const int kb = k / kBlk, ki = k % kBlk;
        float *pbase = part + (size_t)split * A.K * A.C * (S * R);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int c = cg * 64 + ch * 32 + 8 * (r / 4) + 4 * half + (r % 4);
            if (c >= A.C) continue;
            float *p = pbase + ((size_t)kb * CB + c / kBlk) * (S * R * kBlk * kBlk) + (c % kBlk) * kBlk + ki;
#pragma unroll
            for (int tp = 0; tp < S * R; ++tp) p[tp * (kBlk * kBlk)] = acc[tp][r];
        }
    }
}

// ------------------------------------------------------------------------------------------
// 1x1 layers (unit stride, no padding): dw[k][c] = sum over all N*H*W pixels of dy[p][k] * x[p][c],
// a matrix product with the pixels as the reduction dimension (Sec. 5.2 of the paper).  Pixels are
// numbered across the minibatch and cut into chunks of PWP; `units` counts chunks.
// ------------------------------------------------------------------------------------------
constexpr int kPwP = 32;            // pixels per staged chunk

// Dense: workgroup = CW input channels x KW output channels (128 or 64 each), its four wavefronts a 2 x 2
// grid of (CW/2) x (KW/2) sub-tiles of 32x32 MFMA blocks; the next chunk of P pixels is fetched into registers
// while the current one is multiplied.  128 x 128 uses a staged pixel for four MFMAs per pair of LDS reads;
// layers with only 64 channels on a side get the narrower tile (no padded blocks) and chunks of 64 pixels,
// so that there are as many MFMAs between two barriers.
template <int CW, int KW, int P>
__global__ __launch_bounds__(256) void pw_bww_dense_kernel(BwwArgs A, const float *__restrict__ x,
                                                           const float *__restrict__ dy,
                                                           float *__restrict__ part)
{
    if (deselected(A.sel, A.want)) return;              // uniform over the grid, before any barrier
    constexpr int CI = CW / 64, KJ = KW / 64;           // 32x32 blocks per wavefront along c and along k
    constexpr int NX = P * CW / 4 / 256, ND = P * KW / 4 / 256;      // float4 staging slots per thread
    __shared__ __attribute__((aligned(16))) float xs[P * CW];
    __shared__ __attribute__((aligned(16))) float ds[P * KW];

    // the wavefront index is the same in every lane: kept in a scalar register, and with it every tile coordinate
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;
    const int l32 = lane % 32, half = lane / 32;
    const int wk = wave % 2, wc = wave / 2;
    const int split = blockIdx.x;
    const int kt = blockIdx.y / A.cgroups, cg = blockIdx.y % A.cgroups;     // groups of KW / CW channels here
    const int CB = A.C / kBlk, KB = A.K / kBlk;
    const int HW = A.H * A.W;

    floatx16 acc[CI][KJ];                               // [c block of 32][k block of 32]
#pragma unroll
    for (int i = 0; i < CI; ++i)
#pragma unroll
        for (int j = 0; j < KJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int u0 = (int)((long long)A.units * split / A.splits);
    const int u1 = (int)((long long)A.units * (split + 1) / A.splits);

    // staging slots of this thread: slot = (pixel, 4 channels).  (image, pixel) of a chunk's first pixel is
    // carried from chunk to chunk (one 64-bit division per workgroup instead of one per slot and chunk); a
    // slot's pixel is that plus its offset, wrapped into the following images.
    float4 rx[NX], rd[ND];
    int n0 = (int)((long long)u0 * P / HW), p0 = (int)((long long)u0 * P % HW);
    auto locate = [&](int pix, int &n, int &p) __attribute__((always_inline)) {
        n = n0;
        p = p0 + pix;
        while (p >= HW) { p -= HW; ++n; }
        return n < A.N;
    };
    auto fetch = [&]() __attribute__((always_inline)) {      // the chunk that starts at (n0, p0)
#pragma unroll
        for (int jj = 0; jj < NX; ++jj) {
            const int idx = jj * 256 + (int)threadIdx.x;
            const int pix = idx / (CW / 4), q = idx % (CW / 4);
            const int cb = cg * (CW / kBlk) + (q >> 2);
            int n, p;
            rx[jj] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (locate(pix, n, p) && cb < CB)
                rx[jj] = *reinterpret_cast<const float4 *>(x + (((size_t)n * CB + cb) * HW + p) * kBlk + (q & 3) * 4);
        }
#pragma unroll
        for (int jj = 0; jj < ND; ++jj) {
            const int idx = jj * 256 + (int)threadIdx.x;
            const int pix = idx / (KW / 4), q = idx % (KW / 4);
            const int kb = kt * (KW / kBlk) + (q >> 2);
            int n, p;
            rd[jj] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (locate(pix, n, p) && kb < KB)
                rd[jj] = *reinterpret_cast<const float4 *>(dy + (((size_t)n * KB + kb) * HW + p) * kBlk + (q & 3) * 4);
        }
        p0 += P;
        while (p0 >= HW) { p0 -= HW; ++n0; }
    };
    auto stash = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int jj = 0; jj < NX; ++jj) *reinterpret_cast<float4 *>(xs + (jj * 256 + (int)threadIdx.x) * 4) = rx[jj];     // [pixel][CW c]
#pragma unroll
        for (int jj = 0; jj < ND; ++jj) *reinterpret_cast<float4 *>(ds + (jj * 256 + (int)threadIdx.x) * 4) = rd[jj];     // [pixel][KW k]
    };

    if (u0 < u1) fetch();
    for (int unit = u0; unit < u1; ++unit) {
        __syncthreads();                                // the previous chunk is no longer read
        stash();
        __syncthreads();
        if (unit + 1 < u1) fetch();                     // in flight during the MFMAs below
#pragma unroll 4
        for (int pp = 0; pp < P / 2; ++pp) {
            const int p = 2 * pp + half;                // A[i = c][kk = half], B[kk = half][j = k]
            float av[CI], bv[KJ];
#pragma unroll
            for (int i = 0; i < CI; ++i) av[i] = xs[p * CW + wc * (CW / 2) + i * 32 + l32];
#pragma unroll
            for (int j = 0; j < KJ; ++j) bv[j] = ds[p * KW + wk * (KW / 2) + j * 32 + l32];
#pragma unroll
            for (int i = 0; i < CI; ++i)
#pragma unroll
                for (int j = 0; j < KJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
    }

    // D[i = c][j = k]: column = lane % 32, row = 8*(r/4) + 4*(lane/32) + r%4
    float *pbase = part + (size_t)split * A.K * A.C;
#pragma unroll
    for (int j = 0; j < KJ; ++j) {
        const int k = kt * KW + wk * (KW / 2) + j * 32 + l32;
        if (k >= A.K) continue;
#pragma unroll
        for (int i = 0; i < CI; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int c = cg * CW + wc * (CW / 2) + i * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                if (c < A.C)
                    pbase[((size_t)(k / kBlk) * CB + c / kBlk) * (kBlk * kBlk) + (c % kBlk) * kBlk + k % kBlk] = acc[i][j][r];
            }
    }
}

// Zero-skipping: lane = KPL output channels (k, k+64, ...), wavefront = 8 input channels, workgroup =
// 8 wavefronts = 64 input channels, as in bww_sparse_kernel but with KPL accumulators per tested
// element instead of R*S: without taps, the number of multiply-adds a zero saves is the number of
// output channels a lane owns (T = K/64 up to 4), the 1x1 analogue of T = Q/V in Sec. 5.2.
template <int KPL>
__global__ __launch_bounds__(512, 4) void pw_bww_sparse_kernel(BwwArgs A, const float *__restrict__ x,
                                                               const float *__restrict__ dy,
                                                               float *__restrict__ part)
{
    constexpr int P = kPwP, CH = 8, GP = 4, KW = 64 * KPL;
    if (deselected(A.sel, A.want)) return;              // uniform over the grid, before any barrier
    __shared__ __attribute__((aligned(16))) float dyT[P * KW];
    __shared__ __attribute__((aligned(16))) float xT[P * 64];

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int lane = threadIdx.x % kWave;
    const int split = blockIdx.x;
    const int kt = blockIdx.y / A.cgroups, cg = blockIdx.y % A.cgroups;     // kt: groups of KW, cg: of 64
    const int CB = A.C / kBlk, KB = A.K / kBlk;
    const int cbl = wave >> 1, h = wave & 1;
    const int cb = cg * 4 + cbl;
    const bool wave_active = cb < CB;
    const int HW = A.H * A.W;

    float acc[CH][KPL];
#pragma unroll
    for (int ci = 0; ci < CH; ++ci)
#pragma unroll
        for (int j = 0; j < KPL; ++j) acc[ci][j] = 0.f;

    const int u0 = (int)((long long)A.units * split / A.splits);
    const int u1 = (int)((long long)A.units * (split + 1) / A.splits);
    const int mpix = lane >> 4, mch = lane & 15;

    // (image, pixel) of the chunk's first pixel, carried from chunk to chunk: one 64-bit division per
    // workgroup instead of one per staged float4
    int n0 = (int)((long long)u0 * P / HW), p0 = (int)((long long)u0 * P % HW);
    auto locate = [&](int pix, int &n, int &p) __attribute__((always_inline)) {
        n = n0;
        p = p0 + pix;
        while (p >= HW) { p -= HW; ++n; }
        return n < A.N;
    };
    // A thread's 16-byte pieces of a chunk (KPL of dy, one of x; zeros past the last image and beyond the channel
    // count) are asked for while the previous chunk is worked on and written to LDS after it: with load, wait
    // and write in turn a chunk of 32 pixels cost KPL + 1 memory round trips, more than its arithmetic.
    constexpr int NDY = P * (KW / 4) / 512;
    static_assert(NDY * 512 == P * (KW / 4) && P * 16 == 512, "one x piece and KPL dy pieces per thread");
    float4 sdy[NDY], sxv;
    auto fetch = [&]() __attribute__((always_inline)) {
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));                   // (slot arithmetic redone per chunk, not kept in registers)
#pragma unroll
        for (int i = 0; i < NDY; ++i) {
            const int idx = tid + i * 512;
            const int pix = idx / (KW / 4), q = idx % (KW / 4);
            const int kb = kt * (KW / kBlk) + (q >> 2);
            int n, p;
            sdy[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (locate(pix, n, p) && kb < KB)
                sdy[i] = *reinterpret_cast<const float4 *>(dy + (((size_t)n * KB + kb) * HW + p) * kBlk + (q & 3) * 4);
        }
        {
            const int pix = tid >> 4, q = tid & 15;
            const int cbq = cg * 4 + (q >> 2);
            int n, p;
            sxv = make_float4(0.f, 0.f, 0.f, 0.f);
            if (locate(pix, n, p) && cbq < CB)
                sxv = *reinterpret_cast<const float4 *>(x + (((size_t)n * CB + cbq) * HW + p) * kBlk + (q & 3) * 4);
        }
        p0 += P;
        while (p0 >= HW) { p0 -= HW; ++n0; }
    };
    if (u0 < u1) fetch();
    for (int unit = u0; unit < u1; ++unit) {
        __syncthreads();                                // every wavefront is done with the previous chunk
        {
            int tid = threadIdx.x;
            asm volatile("" : "+v"(tid));
#pragma unroll
            for (int i = 0; i < NDY; ++i) *reinterpret_cast<float4 *>(dyT + (tid + i * 512) * 4) = sdy[i];   // = [pix][q*4]
            *reinterpret_cast<float4 *>(xT + tid * 4) = sxv;
        }
        __syncthreads();
        if (unit + 1 < u1) fetch();                     // in flight during this chunk's work
        if (!wave_active) continue;

        // accumulators of channels 2i + 1 and 2i in (even, odd) register pairs, as in bww_sparse_kernel: never
        // the parity of the channel's tested value
        typedef float f2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int ci = 0; ci < CH; ci += 2)
#pragma unroll
            for (int q = 0; q < KPL; ++q) {
                f2 pr = {acc[ci + 1][q], acc[ci][q]};
                asm volatile("" : "+v"(pr));
                acc[ci + 1][q] = pr.x;
                acc[ci][q] = pr.y;
            }

        float mnext = xT[mpix * 64 + cbl * 16 + mch];        // mask values are read one group ahead
        for (int g0 = 0; g0 < P; g0 += GP) {
            const float mval = mnext;
            if (g0 + GP < P) mnext = xT[(g0 + GP + mpix) * 64 + cbl * 16 + mch];
            const unsigned long long m64 = __builtin_amdgcn_ballot_w64(mval != 0.f);
            const unsigned mlo = (unsigned)m64, mhi = (unsigned)(m64 >> 32);
            if ((mlo | mhi) == 0u) continue;
            float dyw[GP][KPL];
#pragma unroll
            for (int j = 0; j < GP; ++j)
#pragma unroll
                for (int q = 0; q < KPL; ++q) dyw[j][q] = dyT[(g0 + j) * KW + q * 64 + lane];
            const float4 *xq = reinterpret_cast<const float4 *>(xT + g0 * 64 + cbl * 16 + h * CH);
            float4 xlo = xq[0], xhi = xq[1];
            __builtin_amdgcn_s_waitcnt(0xC07F);
            static_for<0, GP>([&](auto J) __attribute__((always_inline)) {
                constexpr int j = decltype(J)::value;
                float4 nlo = xlo, nhi = xhi;
                if constexpr (j + 1 < GP) {
                    nlo = xq[(j + 1) * 16];
                    nhi = xq[(j + 1) * 16 + 1];
                }
                const float xv[CH] = {xlo.x, xlo.y, xlo.z, xlo.w, xhi.x, xhi.y, xhi.z, xhi.w};
                const unsigned mw = (j < 2) ? mlo : mhi;
                constexpr int sh = (j % 2) * 16;
                const unsigned bits = (mw >> sh) >> (h * CH) & 0xFFu;
                if (__builtin_expect(bits != 0u, 1)) {
                    static_for<0, CH>([&](auto CI) __attribute__((always_inline)) {
                        constexpr int ci = decltype(CI)::value;
                        if (__builtin_expect((bits & (1u << ci)) != 0u, 1)) {
#pragma unroll
                            for (int q = 0; q < KPL; ++q) acc[ci][q] = fmaf(xv[ci], dyw[j][q], acc[ci][q]);
                        }
                    });
                }
                if constexpr (j + 1 < GP) __builtin_amdgcn_s_waitcnt(0xC07F);
                xlo = nlo;
                xhi = nhi;
            });
        }
    }

    if (wave_active) {
        float *pbase = part + (size_t)split * A.K * A.C;
#pragma unroll
        for (int q = 0; q < KPL; ++q) {
            const int k = kt * KW + q * 64 + lane;
            if (k >= A.K) continue;
            if (!A.swapped) {
                float *p = pbase + ((size_t)(k / kBlk) * CB + cb) * (kBlk * kBlk) + (h * CH) * kBlk + k % kBlk;
#pragma unroll
                for (int ci = 0; ci < CH; ++ci) p[ci * kBlk] = acc[ci][q];
            } else {            // exchanged operands: block [cb][k block] of the layer, element [k % 16][h*8 + ci]
                float4 *p = reinterpret_cast<float4 *>(pbase + ((size_t)cb * KB + k / kBlk) * (kBlk * kBlk) +
                                                       (k % kBlk) * kBlk + h * CH);
                p[0] = make_float4(acc[0][q], acc[1][q], acc[2][q], acc[3][q]);
                p[1] = make_float4(acc[4][q], acc[5][q], acc[6][q], acc[7][q]);
            }
        }
    }
}

// dw[i] = sum over splits of part[s][i].  A workgroup owns 64 float4 outputs; its 16 wavefronts each
// add the splits s = w, w+16, ... (in that order) and wavefront 0 adds the 16 sums in wavefront
// order: a fixed tree, so the result does not depend on timing.  Layers with few filter elements
// and many splits (1x1, 64 x 64) would otherwise leave the sum to a handful of threads.
// dw may be the first partial itself (every element is read by the thread that later writes it).
// The grid is capped and workgroups stride over the outputs: a launch whose form was not selected
// (st_conv_bww_auto) then costs a few hundred workgroup dispatches instead of up to ten thousand.
// sp.f[form] = number of partial sums the form (0 tests x, 1 tests dy, 2 dense) leaves behind; with
// want = kAnyForm the launch adds up those of whichever form the sampled counts selected, else it
// belongs to the form `want` and does nothing when another one was selected.
struct Splits3 { int f[3]; };
constexpr int kAnyForm = -2;
__global__ __launch_bounds__(1024) void bww_reduce_kernel(const float4 *part, float4 *dw, size_t n4, Splits3 sp,
                                                          const unsigned *sel, int want)
{
    int form = want < 0 ? 0 : want;
    if (sel) {
        form = selected_form(sel);
        if (want != kAnyForm && form != want) return;
    }
    const int splits = form == 0 ? sp.f[0] : form == 1 ? sp.f[1] : sp.f[2];
    __shared__ float4 red[16][64];
    const int o = threadIdx.x % 64, sl = threadIdx.x / 64;
    const size_t nblk = (n4 + 63) / 64;
    for (size_t blk = blockIdx.x; blk < nblk; blk += gridDim.x) {       // uniform trip count per workgroup
        const size_t i = blk * 64 + o;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i < n4)
            for (int p = sl; p < splits; p += 16) {
                const float4 v = part[(size_t)p * n4 + i];
                s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
            }
        red[sl][o] = s;
        __syncthreads();
        if (sl == 0 && i < n4) {
            const int lanes = splits < 16 ? splits : 16;
            for (int q = 1; q < lanes; ++q) {
                const float4 v = red[q][o];
                s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
            }
            dw[i] = s;
        }
        __syncthreads();                                    // red is rewritten by the next round
    }
}

constexpr size_t kReduceGrid = 512;          // workgroups of 1024 threads: two per compute unit
constexpr int kSparseTH = 7, kSparseTW = 8;     // unit stride: 224 ... 7 are multiples of 7; two double-buffered workgroups fit the LDS
constexpr int kSparseS2TH = 8, kSparseS2TW = 8; // stride 2, x tested
constexpr size_t kSparseLds = bww_async_lds_bytes<3, 3, kSparseTH, kSparseTW>();

// The zero-skipping unit-stride kernels use more dynamic LDS than a kernel may without being allowed to: once per
// device, outside any launch sequence a caller may be capturing into a graph later.
template <class K>
hipError_t allow_dynamic_lds(K kern, size_t bytes)
{
    constexpr int kMaxDev = 64;
    static bool allowed[kMaxDev] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDev) return hipErrorInvalidDevice;
    if (!allowed[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return e;
        allowed[dev] = true;
    }
    return hipSuccess;
}
BwwArgs make_args(const st_conv_desc &d, int TH, int TW, bool tiles_over_input);
BwwArgs sparse_args(const st_conv_desc &d);
BwwArgs dense_args(const st_conv_desc &d);
bool dense_narrow(const st_conv_desc &d);
bool bww_s2(const st_conv_desc &d);
constexpr int kDenseTH = 7, kDenseTW = 14;   // 224, 112, 56, 28 and 14 are multiples of both: no ragged tiles
constexpr int kDenseNarrowTW = 8;            // output rows of at most 8 pixels (7 x 7 layers): half of a 14-wide tile would be padding
// stride-2 layers: 4x8 tiles keep the strided halo of the other operand (9x17 pixels x 64 channels) in LDS
constexpr int kS2TH = 4, kS2TW = 8;

constexpr int kBwwTargetWorkgroups = 512;

BwwArgs make_args(const st_conv_desc &d, int TH, int TW, bool tiles_over_input)
{
    BwwArgs A;
    A.sel = nullptr; A.want = 0; A.swapped = 0;
    A.N = d.N; A.C = d.C; A.K = d.K; A.H = d.H; A.W = d.W;
    A.OH = (d.H + 2 * d.pad_h - d.S) / d.stride_h + 1;
    A.OW = (d.W + 2 * d.pad_w - d.R) / d.stride_w + 1;
    A.pw = d.pad_w; A.ph = d.pad_h;
    const int eh = tiles_over_input ? d.H : A.OH, ew = tiles_over_input ? d.W : A.OW;
    A.tiles_h = ceil_div(eh, TH);
    A.tiles_w = ceil_div(ew, TW);
    A.units = d.N * A.tiles_h * A.tiles_w;
    A.cgroups = ceil_div(d.C, 64);
    const int groups = ceil_div(d.K, 64) * A.cgroups;
    // number of partial sums: enough workgroups to fill the chip (256 compute units, 2 resident
    // workgroups each)
    int splits = ceil_div(kBwwTargetWorkgroups, groups);
    if (splits > A.units) splits = A.units;
    if (splits < 1) splits = 1;
    A.splits = splits;
    return A;
}

// tiles of the dense unit-stride 3x3 kernel
bool dense_narrow(const st_conv_desc &d) { return d.W + 2 * d.pad_w - d.R + 1 <= kDenseNarrowTW; }
BwwArgs dense_args(const st_conv_desc &d)
{
    return make_args(d, kDenseTH, dense_narrow(d) ? kDenseNarrowTW : kDenseTW, false);
}

// tiles of the zero-skipping 3x3 kernel that tests the input of layer d
BwwArgs sparse_args(const st_conv_desc &d)
{
    return bww_s2(d) ? make_args(d, kSparseS2TH, kSparseS2TW, true) : make_args(d, kSparseTH, kSparseTW, true);
}

// 1x1 layers: chunks of kPwP pixels numbered across the minibatch; kw / cw = channels per workgroup
BwwArgs make_args_pw(const st_conv_desc &d, int kw, int cw, int chunk = kPwP, int target = kBwwTargetWorkgroups)
{
    BwwArgs A;
    A.sel = nullptr; A.want = 0; A.swapped = 0;
    A.N = d.N; A.C = d.C; A.K = d.K; A.H = d.H; A.W = d.W; A.OH = d.H; A.OW = d.W; A.pw = 0; A.ph = 0;
    A.tiles_h = A.tiles_w = 1;
    const long long chunks = ((long long)d.N * d.H * d.W + chunk - 1) / chunk;
    A.units = (int)chunks;                          // bww_fast_supported bounds N*H*W
    A.cgroups = ceil_div(d.C, cw);
    const int groups = ceil_div(d.K, kw) * A.cgroups;
    int splits = ceil_div(target, groups);
    if (splits > A.units) splits = A.units;
    if (splits < 1) splits = 1;
    A.splits = splits;
    return A;
}

// dense 1x1 BWW: channels of one operand per workgroup (128, or 64 for layers with no more than that), and the
// pixels per staged chunk that go with the tile
int pw_dense_tile(int channels) { return channels > 64 ? 128 : 64; }
constexpr int kPwDenseWorkgroups = 512;         // two per compute unit: measured best of 256 / 512 / 1024
BwwArgs make_args_pw_dense(const st_conv_desc &d)
{
    const int cw = pw_dense_tile(d.C), kw = pw_dense_tile(d.K);
    return make_args_pw(d, kw, cw, cw == 128 && kw == 128 ? 32 : 64, kPwDenseWorkgroups);
}

int pw_kpl(const st_conv_desc &d) { return d.K % 256 == 0 ? 4 : (d.K % 128 == 0 ? 2 : 1); }

size_t partial_bytes(const st_conv_desc &d, const BwwArgs &A)
{
    if (A.splits == 1) return 0;
    return (size_t)A.splits * d.K * d.C * d.S * d.R * sizeof(float);
}

hipError_t reduce(const st_conv_desc &d, const BwwArgs &A, const float *part, float *dw, hipStream_t s)
{
    if (A.splits == 1) return hipSuccess;               // the kernel wrote dw itself
    const size_t n4 = (size_t)d.K * d.C * d.S * d.R / 4;
    const size_t nblk = (n4 + 63) / 64;
    const int form = A.sel ? A.want : 0;
    Splits3 sp = {{A.splits, A.splits, A.splits}};
    hipLaunchKernelGGL(bww_reduce_kernel, dim3((unsigned)(nblk < kReduceGrid ? nblk : kReduceGrid)), dim3(1024), 0, s,
                       reinterpret_cast<const float4 *>(part), reinterpret_cast<float4 *>(dw), n4, sp, A.sel, form);
    return hipGetLastError();
}

}  // namespace

namespace {
bool bww_s2(const st_conv_desc &d)
{
    return d.stride_w == 2 && d.stride_h == 2 && d.R == 3 && d.S == 3 && d.pad_w == 1 && d.pad_h == 1;
}

// stride 2, dy tested: the tested tile runs over dy (OH x OW, K channels), the halo over x
BwwArgs make_args_s2_dy(const st_conv_desc &d)
{
    st_conv_desc e = d;
    e.C = d.K; e.K = d.C;
    e.H = (d.H + 2 * d.pad_h - d.S) / 2 + 1;
    e.W = (d.W + 2 * d.pad_w - d.R) / 2 + 1;
    e.stride_w = e.stride_h = 1;
    BwwArgs A = make_args(e, kS2TH, kS2TW, true);
    A.OH = d.H; A.OW = d.W;                         // size of the halo operand (x)
    A.pw = d.pad_w; A.ph = d.pad_h;
    return A;
}
}  // namespace

bool bww_fast_supported(const st_conv_desc &d)
{
    // gridDim.y carries (output-channel group, input-channel group), at least 32 channels each, with
    // either operand in either role
    if ((long long)ceil_div(d.K, 32) * ceil_div(d.C, 32) > 65535) return false;
    if (bww_s2(d)) return (long long)d.N * ceil_div(d.H, 4) * ceil_div(d.W, 8) <= 0x7fffffffLL;
    if (d.stride_w != 1 || d.stride_h != 1) return false;
    const long long units = (long long)d.N * ceil_div(d.H + 2 * d.pad_h, 7) * ceil_div(d.W + 2 * d.pad_w, 8);
    if (units > 0x7fffffffLL) return false;
    if (d.R == 3 && d.S == 3) return d.pad_w <= 2 && d.pad_h <= 2;
    if (d.R == 1 && d.S == 1)
        return d.pad_w == 0 && d.pad_h == 0 && (long long)d.N * d.H * d.W / kPwP < 0x7fffff00LL;
    return false;
}

size_t bww_sparse_workspace(const st_conv_desc &d)
{
    if (d.R == 1 && d.S == 1) return partial_bytes(d, make_args_pw(d, 64 * pw_kpl(d), 64));
    return partial_bytes(d, sparse_args(d));
}

size_t bww_dense_workspace(const st_conv_desc &d)
{
    if (d.R == 1 && d.S == 1) return partial_bytes(d, make_args_pw_dense(d));
    if (bww_s2(d)) return partial_bytes(d, make_args(d, kS2TH, kS2TW, false));
    return partial_bytes(d, dense_args(d));
}

namespace {
// e = the layer as the kernel sees it (e.C tested channels, e.K lane channels); swapped = dy tested:
// the partial sums are then dw'[c][k] and go through the transposing reduction
hipError_t launch_pw_sparse(const st_conv_desc &d, const st_conv_desc &e, const float *tested, const float *other,
                            float *dw, float *ws, bool swapped, hipStream_t s, const unsigned *sel)
{
    const int kpl = pw_kpl(e);
    BwwArgs A = make_args_pw(e, 64 * kpl, 64);
    A.sel = sel; A.want = swapped ? 1 : 0; A.swapped = swapped ? 1 : 0;
    float *part = A.splits == 1 ? dw : ws;
    dim3 grid(A.splits, ceil_div(e.K, 64 * kpl) * A.cgroups);
    if (kpl == 4) hipLaunchKernelGGL(pw_bww_sparse_kernel<4>, grid, dim3(512), 0, s, A, tested, other, part);
    else if (kpl == 2) hipLaunchKernelGGL(pw_bww_sparse_kernel<2>, grid, dim3(512), 0, s, A, tested, other, part);
    else hipLaunchKernelGGL(pw_bww_sparse_kernel<1>, grid, dim3(512), 0, s, A, tested, other, part);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    return reduce(d, A, part, dw, s);
}
}  // namespace

// name of the kernel instance launch_bww_sparse runs for d (requires bww_fast_supported(d))
void bww_sparse_kernel_name(const st_conv_desc &d, char *buf, size_t len)
{
    if (d.R == 1) snprintf(buf, len, "pw_bww_sparse_kernel<%d>", pw_kpl(d));
    else if (bww_s2(d)) snprintf(buf, len, "bww_sparse_kernel<3, 3, %d, %d, 1>", kSparseS2TH, kSparseS2TW);
    else snprintf(buf, len, "bww_sparse_kernel<3, 3, %d, %d, 0>", kSparseTH, kSparseTW);
}

hipError_t launch_bww_sparse(const st_conv_desc &d, const float *x, const float *dy, float *dw,
                             float *ws, hipStream_t s, const unsigned *sel)
{
    if (d.R == 1) return launch_pw_sparse(d, d, x, dy, dw, ws, false, s, sel);
    BwwArgs A = sparse_args(d);
    A.sel = sel; A.want = 0;
    float *part = A.splits == 1 ? dw : ws;
    dim3 grid(A.splits, ceil_div(d.K, 64) * A.cgroups);
    if (bww_s2(d)) {
        hipLaunchKernelGGL((bww_sparse_kernel<3, 3, kSparseS2TH, kSparseS2TW, 1>), grid, dim3(512), 0, s, A, x, dy, part);
        hipError_t err = hipGetLastError();
        return err != hipSuccess ? err : reduce(d, A, part, dw, s);
    }
    hipError_t e = allow_dynamic_lds(bww_sparse_kernel<3, 3, kSparseTH, kSparseTW, 0>, kSparseLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((bww_sparse_kernel<3, 3, kSparseTH, kSparseTW, 0>), grid, dim3(512), kSparseLds, s, A, x, dy, part);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return reduce(d, A, part, dw, s);
}

// BWW that tests dy: the same kernel with the operand roles exchanged.  With unit stride,
//   dw[k,c,v,u] = sum x[n,c,oh-ph+v,ow-pw+u] dy[n,k,oh,ow] = sum dy[n,k,ih-ph'+v',iw-pw'+u'] x[n,c,ih,iw]
// for v' = S-1-v, ph' = S-1-ph (same for the width), i.e. the filter gradient of a layer whose
// input is dy (K channels, OH x OW, padding S-1-pad) and whose output gradient is x (C channels).
namespace {
st_conv_desc swapped_desc(const st_conv_desc &d)
{
    st_conv_desc e = d;
    e.C = d.K; e.K = d.C;
    e.H = d.H + 2 * d.pad_h - d.S + 1;
    e.W = d.W + 2 * d.pad_w - d.R + 1;
    e.pad_h = d.S - 1 - d.pad_h;
    e.pad_w = d.R - 1 - d.pad_w;
    return e;
}
}  // namespace

bool bww_dy_fast_supported(const st_conv_desc &d)
{
    if (bww_s2(d)) return bww_fast_supported(d);
    return bww_fast_supported(d) && d.pad_h <= d.S - 1 && d.pad_w <= d.R - 1 && bww_fast_supported(swapped_desc(d));
}

size_t bww_sparse_dy_workspace(const st_conv_desc &d)
{
    if (d.R == 1 && d.S == 1) {
        const st_conv_desc e = swapped_desc(d);
        return (size_t)make_args_pw(e, 64 * pw_kpl(e), 64).splits * d.K * d.C * sizeof(float);
    }
    if (bww_s2(d)) return (size_t)make_args_s2_dy(d).splits * d.K * d.C * d.S * d.R * sizeof(float);
    const st_conv_desc e = swapped_desc(d);
    const BwwArgs A = make_args(e, kSparseTH, kSparseTW, true);
    return (size_t)A.splits * d.K * d.C * d.S * d.R * sizeof(float);
}

hipError_t launch_bww_sparse_dy(const st_conv_desc &d, const float *x, const float *dy, float *dw,
                                float *ws, hipStream_t s, const unsigned *sel)
{
    if (bww_s2(d)) {
        BwwArgs A = make_args_s2_dy(d);
        A.sel = sel; A.want = 1; A.swapped = 1;
        float *part = A.splits == 1 ? dw : ws;
        dim3 grid(A.splits, ceil_div(A.K, 64) * A.cgroups);
        hipLaunchKernelGGL((bww_sparse_kernel<3, 3, kS2TH, kS2TW, 2>), grid, dim3(512), 0, s, A, dy, x, part);
        hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
        return reduce(d, A, part, dw, s);
    }
    const st_conv_desc e = swapped_desc(d);
    if (d.R == 1) return launch_pw_sparse(d, e, dy, x, dw, ws, true, s, sel);
    BwwArgs A = make_args(e, kSparseTH, kSparseTW, true);
    A.sel = sel; A.want = 1; A.swapped = 1;
    float *part = A.splits == 1 ? dw : ws;
    dim3 grid(A.splits, ceil_div(e.K, 64) * A.cgroups);
    hipError_t err = allow_dynamic_lds(bww_sparse_kernel<3, 3, kSparseTH, kSparseTW, 0>, kSparseLds);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL((bww_sparse_kernel<3, 3, kSparseTH, kSparseTW, 0>), grid, dim3(512), kSparseLds, s, A, dy, x, part);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
    return reduce(d, A, part, dw, s);
}

// st_conv_bww_auto on unit-stride 3x3 layers: one zero-skipping launch that carries the arguments of both
// operand roles and computes the selected one, the dense launch, and one launch that adds up the partial
// sums of whichever form ran.  All three forms stage their partial sums in ws (also a single one).
bool bww_auto_merged_supported(const st_conv_desc &d)
{
    return d.R == 3 && d.S == 3 && d.stride_w == 1 && d.stride_h == 1 && bww_fast_supported(d) && bww_dy_fast_supported(d);
}

hipError_t launch_bww_auto_merged(const st_conv_desc &d, const float *x, const float *dy, float *dw, float *ws,
                                  hipStream_t s, const unsigned *sel)
{
    const st_conv_desc e = swapped_desc(d);
    BwwArgs A0 = make_args(d, kSparseTH, kSparseTW, true), A1 = make_args(e, kSparseTH, kSparseTW, true);
    BwwArgs A2 = dense_args(d);
    A0.sel = A1.sel = A2.sel = sel;
    A0.want = kEitherOperand; A1.want = kEitherOperand; A1.swapped = 1; A2.want = 2;
    const int ygroups = ceil_div(d.K, 64) * ceil_div(d.C, 64);      // the same for both operand roles
    dim3 grid(A0.splits > A1.splits ? A0.splits : A1.splits, ygroups);
    hipError_t err = allow_dynamic_lds(bww_sparse_either_kernel<3, 3, kSparseTH, kSparseTW>, kSparseLds);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL((bww_sparse_either_kernel<3, 3, kSparseTH, kSparseTW>), grid, dim3(512), kSparseLds, s, A0, A1, x, dy, ws);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (dense_narrow(d)) hipLaunchKernelGGL((bww_dense_kernel<3, 3, kDenseTH, kDenseNarrowTW>), dim3(A2.splits, ygroups), dim3(256), 0, s, A2, x, dy, ws);
    else hipLaunchKernelGGL((bww_dense_kernel<3, 3, kDenseTH, kDenseTW>), dim3(A2.splits, ygroups), dim3(256), 0, s, A2, x, dy, ws);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    const size_t n4 = (size_t)d.K * d.C * d.S * d.R / 4;
    const size_t nblk = (n4 + 63) / 64;
    Splits3 sp = {{A0.splits, A1.splits, A2.splits}};
    hipLaunchKernelGGL(bww_reduce_kernel, dim3((unsigned)(nblk < kReduceGrid ? nblk : kReduceGrid)), dim3(1024), 0, s,
                       reinterpret_cast<const float4 *>(ws), reinterpret_cast<float4 *>(dw), n4, sp, sel, kAnyForm);
    return hipGetLastError();
}

hipError_t launch_bww_dense(const st_conv_desc &d, const float *x, const float *dy, float *dw,
                            float *ws, hipStream_t s, const unsigned *sel)
{
    if (bww_s2(d)) {
        BwwArgs A2 = make_args(d, kS2TH, kS2TW, false);
        A2.sel = sel; A2.want = 2;
        dim3 grid2(A2.splits, ceil_div(d.K, 64) * A2.cgroups);
        hipLaunchKernelGGL((bww_dense_kernel<3, 3, kS2TH, kS2TW, 2>), grid2, dim3(256), 0, s, A2, x, dy,
                           A2.splits == 1 ? dw : ws);
        hipError_t err = hipGetLastError();
        return err != hipSuccess ? err : reduce(d, A2, ws, dw, s);
    }
    if (d.R == 1) {
        BwwArgs A1 = make_args_pw_dense(d);
        A1.sel = sel; A1.want = 2;
        const int cw = pw_dense_tile(d.C), kw = pw_dense_tile(d.K);
        dim3 grid1(A1.splits, ceil_div(d.K, kw) * A1.cgroups);
        float *part1 = A1.splits == 1 ? dw : ws;
        if (cw == 128 && kw == 128) hipLaunchKernelGGL((pw_bww_dense_kernel<128, 128, 32>), grid1, dim3(256), 0, s, A1, x, dy, part1);
        else if (cw == 128) hipLaunchKernelGGL((pw_bww_dense_kernel<128, 64, 64>), grid1, dim3(256), 0, s, A1, x, dy, part1);
        else if (kw == 128) hipLaunchKernelGGL((pw_bww_dense_kernel<64, 128, 64>), grid1, dim3(256), 0, s, A1, x, dy, part1);
        else hipLaunchKernelGGL((pw_bww_dense_kernel<64, 64, 64>), grid1, dim3(256), 0, s, A1, x, dy, part1);
        hipError_t err = hipGetLastError();
        return err != hipSuccess ? err : reduce(d, A1, ws, dw, s);
    }
    BwwArgs A = dense_args(d);
    A.sel = sel; A.want = 2;
    float *part = A.splits == 1 ? dw : ws;
    dim3 grid(A.splits, ceil_div(d.K, 64) * A.cgroups);
    if (dense_narrow(d)) hipLaunchKernelGGL((bww_dense_kernel<3, 3, kDenseTH, kDenseNarrowTW>), grid, dim3(256), 0, s, A, x, dy, part);
    else hipLaunchKernelGGL((bww_dense_kernel<3, 3, kDenseTH, kDenseTW>), grid, dim3(256), 0, s, A, x, dy, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return reduce(d, A, part, dw, s);
}

// Measured on the layer shapes of the paper's Table 1: the 3x3 zero-skipping forms pass the dense one at
// 20-25 % zeros; a 1x1 layer saves at most K/64 (or C/64) multiply-adds per zero and stays behind the
// matrix cores at every zero fraction measured (up to 95 %): never (1001).  (Stride-2 layers never get
// here: their dy-testing form beats the dense one even without zeros.)
unsigned bww_sparse_threshold(const st_conv_desc &d)
{
    if (!bww_fast_supported(d)) return 0;           // generic kernels: the test only ever removes work
    return d.R == 1 ? 1001 : 250;
}

}  // namespace st
