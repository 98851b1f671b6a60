// The dense matrix-core kernel of the unit-stride correlation as a template (FwdDenseCfg, fwd_dense_body,
// fwd_dense_kernel) and the tiling choices of its launches, for the files that instantiate it.
#pragma once
#include "st_common.hpp"

namespace st {
namespace {

// TWD = tile width: 8 (8 rows), 14 (4 rows) or 28 (2 rows); a tile holds at most 64 pixels, i.e.
// two 32-row MFMA blocks; with 14 or 28 columns the last 8 rows of the second block are padding.
//
// MODE selects how tile pixels, taps and input samples relate:
//   0  unit stride: tile pixel (ty,tx), tap (v,u) reads halo pixel (ty+v, tx+u).
//   1  stride 2 (FWD of the stride-2 3x3 layers): halo pixel (2*ty+v, 2*tx+u).
//   2  BWI of a stride-2 3x3 layer with padding 1, one launch per parity class (PI,PJ) of the dx
//      positions: the tile is an 8x8 (or 4x14, 2x28) block of the positions (2*i+PI, 2*j+PJ); only
//      the taps whose grid position holds a dy sample contribute (SparseTrain Sec. 3.3): for PI = 0
//      the middle tap reading dy row i, for PI = 1 the outer taps reading dy rows i and i+1; the
//      same along the width.  1, 2, 2 and 4 taps for the four classes instead of 9.
template <int R, int S, int TWD, int MODE = 0, int PI = 0, int PJ = 0>
struct FwdDenseCfg {
    static constexpr int TW = TWD, TH = 64 / TWD, NPIX = TH * TW;
    static constexpr int PSTEP = MODE == 1 ? 2 : 1;                 // halo pixels between neighbouring tile pixels
    static constexpr int NV = MODE == 2 ? (PI ? 2 : 1) : S, NU = MODE == 2 ? (PJ ? 2 : 1) : R, NT = NV * NU;
    static constexpr int HH = MODE == 2 ? TH + PI : (TH - 1) * PSTEP + S;
    static constexpr int HW = MODE == 2 ? TW + PJ : (TW - 1) * PSTEP + R;
    static constexpr int HP = HH * HW;
    // tap t = (kv, ku): halo offset (dv, du) and index of the filter tap in the reformatted copy
    static constexpr int dv(int t) { return t / NU; }
    static constexpr int du(int t) { return t % NU; }
    static constexpr int fv(int t) { return MODE == 2 ? (PI ? 2 * (t / NU) : 1) : t / NU; }
    static constexpr int fu(int t) { return MODE == 2 ? (PJ ? 2 * (t % NU) : 1) : t % NU; }
    static constexpr int ftap(int t) { return fv(t) * R + fu(t); }
    // wavefronts per SIMD the register allocator should aim for: 4, or what the LDS of the
    // workgroups (two halo buffers per pixel tile, 160 KB per compute unit) leaves room for
    static constexpr int minw(int kq)
    {
        const int fit = 163840 / (2 * (4 / kq) * BUF * 4);
        return fit >= 4 ? 4 : (fit >= 1 ? fit : 1);
    }
    static constexpr int XST = 20;                  // floats per staged pixel (16 channels + 4 pad)
    static constexpr int BUF = ((HP * XST + 63) / 64) * 64;   // floats per halo buffer
};

// KQ = column blocks (of 32 output channels) per workgroup: 1, 2 or 4; TQ = 4/KQ pixel tiles.
// wg = index of the workgroup among those of the launch, cshare = its share of the channel split;
// lds_base: 2 * TQ halo buffers of BUF floats (fwd_dense_lds_floats), 16-byte aligned.  Every thread of
// the workgroup makes the call (the body contains barriers).
template <int R, int S, int KQ, int TWD, int MODE = 0, int PI = 0, int PJ = 0>
constexpr int fwd_dense_lds_floats() { return 2 * (4 / KQ) * FwdDenseCfg<R, S, TWD, MODE, PI, PJ>::BUF; }

template <int R, int S, int KQ, int TWD, int MODE = 0, int PI = 0, int PJ = 0>
__device__ __forceinline__ void fwd_dense_body(const Geom &g, const float *__restrict__ in, const float *__restrict__ wd,
                                               float *__restrict__ out, int tiles_w, int tiles_h, int kgroups,
                                               int total_tiles, int csplit, size_t part_stride, int wg, int cshare,
                                               float *lds_base)
{
    using Cfg = FwdDenseCfg<R, S, TWD, MODE, PI, PJ>;
    constexpr int TH = Cfg::TH, TW = Cfg::TW, HW = Cfg::HW, HP = Cfg::HP, XST = Cfg::XST, BUF = Cfg::BUF;
    constexpr int TAPS = S * R, TQ = 4 / KQ, NPIX = Cfg::NPIX, NT = Cfg::NT, PSTEP = Cfg::PSTEP;
    constexpr int NLD = (HP * 4 + KQ * 64 - 1) / (KQ * 64);      // float4 loads per lane and block

    // the wavefront index is the same in every lane: kept in a scalar register, and with it every tile coordinate
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;
    const int kqi = wave % KQ, tqi = wave / KQ;
    const int kg = wg % kgroups, tg = wg / kgroups;
    const int tile = tg * TQ + tqi;
    const bool tile_ok = tile < total_tiles;
    int t = tile_ok ? tile : 0;
    const int tw = t % tiles_w; t /= tiles_w;
    const int th = t % tiles_h;
    const int n = t / tiles_h;
    const int oh0 = th * TH, ow0 = tw * TW;         // MODE 2: in units of the parity class's own grid
    const int ih0 = MODE == 2 ? oh0 : oh0 * PSTEP - g.ph, iw0 = MODE == 2 ? ow0 : ow0 * PSTEP - g.pw;
    const int CiB = g.Ci / kBlk, KoB = g.Ko / kBlk;
    // channel split (launches with few tiles): share cshare reduces its part of the channel blocks
    // into its own partial output, which sum_partials_kernel adds up afterwards
    const int cb0 = cshare * (CiB / csplit), cb1 = cb0 + CiB / csplit;            // CiB % csplit == 0
    out += cshare * part_stride;
    const int kb32 = kg * KQ + kqi;                 // this wavefront's column block
    const bool k_ok = kb32 * 32 < g.Ko;
    const bool active = tile_ok && k_ok;

    const int l32 = lane % 32, half = lane / 32;

    floatx16 acc[2];
#pragma unroll
    for (int pb = 0; pb < 2; ++pb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[pb][r] = 0.f;

    // B operand: lane supplies filter element (k = kb32*32 + l32, c = j + 8*half), j = 0..7, from
    // the reformatted copy: element offset (kb32*CiB*TAPS + step)*512 + half*256 + l32*8 + j
    const float *bbase = wd + (size_t)(k_ok ? kb32 : 0) * CiB * TAPS * 512 + half * 256 + l32 * 8;
    auto load_b = [&](int s, float (&b)[8]) __attribute__((always_inline)) {
        const float4 *p = reinterpret_cast<const float4 *>(bbase + (size_t)s * 512);
        const float4 lo = p[0], hi = p[1];
        b[0] = lo.x; b[1] = lo.y; b[2] = lo.z; b[3] = lo.w;
        b[4] = hi.x; b[5] = hi.y; b[6] = hi.z; b[7] = hi.w;
    };
    // A operand: lane supplies input (pixel = pb*32 + l32 of the tile, channels half*8 .. half*8+7)
    int apix[2];
#pragma unroll
    for (int pb = 0; pb < 2; ++pb) {
        const int p = min(pb * 32 + l32, NPIX - 1);        // padding rows read a valid pixel; never stored
        apix[pb] = (p / TW) * PSTEP * HW + (p % TW) * PSTEP;
    }

    // halo staging: the KQ wavefronts of a tile split its HP*4 float4 among their KQ*64 lanes
    const int sl = kqi * kWave + lane;
    auto load_halo = [&](int cb, float4 (&h)[NLD]) __attribute__((always_inline)) {
#pragma unroll
        for (int jj = 0; jj < NLD; ++jj) {
            const int idx = jj * (KQ * kWave) + sl;
            const int pix = idx >> 2, q = idx & 3;
            const int a = pix / HW, b = pix % HW;
            const int ih = ih0 + a, iw = iw0 + b;
            h[jj] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (tile_ok && pix < HP && ih >= 0 && ih < g.Hi && iw >= 0 && iw < g.Wi)
                h[jj] = *reinterpret_cast<const float4 *>(in + act_off(n, cb, ih, iw, CiB, g.Hi, g.Wi) + q * 4);
        }
    };
    auto store_halo = [&](float *buf, const float4 (&h)[NLD]) __attribute__((always_inline)) {
#pragma unroll
        for (int jj = 0; jj < NLD; ++jj) {
            const int idx = jj * (KQ * kWave) + sl;
            const int pix = idx >> 2, q = idx & 3;
            if (pix < HP) *reinterpret_cast<float4 *>(buf + pix * XST + q * 4) = h[jj];
        }
    };

    constexpr int kWaitOlder = vmcnt_imm(2);          // all but the 2 newest loads
    float bcur[8], bnxt[8];
    float4 hreg[NLD];
    load_halo(cb0, hreg);
    store_halo(lds_base + tqi * BUF, hreg);
    load_b(cb0 * TAPS + Cfg::ftap(0), bcur);
    __syncthreads();

    for (int cb = cb0; cb < cb1; ++cb) {
        const float *lds = lds_base + (((cb - cb0) & 1) * TQ + tqi) * BUF;
#pragma unroll
        for (int tp = 0; tp < NT; ++tp) {
            {
                const int v = Cfg::dv(tp), u = Cfg::du(tp);
                // next step's filters fly during this step's MFMAs (the last step re-reads its own)
                const int nstep = tp + 1 < NT ? cb * TAPS + Cfg::ftap(tp + 1 < NT ? tp + 1 : 0)
                                              : min(cb + 1, cb1 - 1) * TAPS + Cfg::ftap(0);
                load_b(nstep, bnxt);
                __builtin_amdgcn_sched_barrier(0);              // keep these loads ahead of the MFMAs below
                float a[2][8];
#pragma unroll
                for (int pb = 0; pb < 2; ++pb) {
                    const float *p = lds + (apix[pb] + v * HW + u) * XST + half * 8;
                    const float4 lo = *reinterpret_cast<const float4 *>(p);
                    const float4 hi = *reinterpret_cast<const float4 *>(p + 4);
                    a[pb][0] = lo.x; a[pb][1] = lo.y; a[pb][2] = lo.z; a[pb][3] = lo.w;
                    a[pb][4] = hi.x; a[pb][5] = hi.y; a[pb][6] = hi.z; a[pb][7] = hi.w;
                }
                __builtin_amdgcn_s_waitcnt(kWaitOlder);         // bcur (and anything older) has arrived
                __builtin_amdgcn_sched_barrier(0);
                // The next block's halo is requested here, after the wait, so that the first wait
                // that covers these loads is the one of the next tap: they land during the MFMAs.
                if (tp == 0 && cb + 1 < cb1) {
                    load_halo(cb + 1, hreg);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (active) {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
#pragma unroll
                        for (int pb = 0; pb < 2; ++pb)
                            acc[pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[pb][j], bcur[j], acc[pb], 0, 0, 0);
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) bcur[j] = bnxt[j];
            }
        }
        if (cb + 1 < cb1) store_halo(lds_base + (((cb + 1 - cb0) & 1) * TQ + tqi) * BUF, hreg);
        __syncthreads();
    }

    // D layout of the 32x32 block: column = lane % 32, row = 8*(r/4) + 4*(lane/32) + r%4
    const int k = kb32 * 32 + l32;
    if (active && k < g.Ko) {
        const int kb = k / kBlk, ki = k % kBlk;
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int p = pb * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                const int oh = MODE == 2 ? 2 * (oh0 + p / TW) + PI : oh0 + p / TW;
                const int ow = MODE == 2 ? 2 * (ow0 + p % TW) + PJ : ow0 + p % TW;
                if (p < NPIX && oh < g.Ho && ow < g.Wo)
                    out[act_off(n, kb, oh, ow, KoB, g.Ho, g.Wo) + ki] = acc[pb][r];
            }
    }
}

template <int R, int S, int KQ, int TWD, int MODE = 0, int PI = 0, int PJ = 0>
__global__ __launch_bounds__(256, (FwdDenseCfg<R, S, TWD, MODE, PI, PJ>::minw(KQ))) void fwd_dense_kernel(
    Geom g, const float *__restrict__ in, const float *__restrict__ wd, float *__restrict__ out, int tiles_w, int tiles_h,
    int kgroups, int total_tiles, int csplit, size_t part_stride)
{
    if (form_deselected(g.sel, g.want, g.thr)) return;
    __shared__ __attribute__((aligned(16))) float lds_all[fwd_dense_lds_floats<R, S, KQ, TWD, MODE, PI, PJ>()];
    fwd_dense_body<R, S, KQ, TWD, MODE, PI, PJ>(g, in, wd, out, tiles_w, tiles_h, kgroups, total_tiles, csplit, part_stride,
                                                 (int)blockIdx.x, (int)blockIdx.y, lds_all);
}

// Tile width and column blocks per workgroup of a unit-stride launch (the choice launch_rs and
// launch_kq make), and the number of workgroups that results
inline void dense_tiling(const Geom &g, int *twd, int *kq, long long *blocks)
{
    // tile width that divides the row length, if any: 8 -> 8x8, 28 -> 2x28, 14 -> 4x14
    *twd = (g.Wo % 8 != 0 && g.Wo % 28 == 0 && g.Ho % 2 == 0) ? 28
         : (g.Wo % 8 != 0 && g.Wo % 14 == 0 && g.Ho % 4 <= g.Ho % 8) ? 14 : 8;
    *kq = g.Ko > 64 ? 4 : (g.Ko > 32 ? 2 : 1);
    const long long tiles = (long long)ceil_div(g.Wo, *twd) * ceil_div(g.Ho, 64 / *twd) * g.N;
    const int tq = 4 / *kq;
    *blocks = (tiles + tq - 1) / tq * ceil_div(g.Ko, 32 * *kq);
}

// Channel split of the unit-stride 3x3 launches that would leave most of the chip idle (7x7 and 14x14
// layers: a workgroup per pixel tile and 128 output channels gives 128 workgroups for 512 -> 512 @7,
// N = 32, each walking all 512 input channels): 2, 4 or 8 shares, enough for about two workgroups per
// compute unit.  Depends on the geometry only, so that the workspace query and the launch agree.
inline int dense_channel_split(const Geom &g)
{
    if (g.R != 3 || g.S != 3 || g.sw != 1 || g.uw != 1) return 1;
    int twd, kq;
    long long blocks;
    dense_tiling(g, &twd, &kq, &blocks);
    if (blocks >= 384) return 1;
    const int CiB = g.Ci / kBlk;
    int cs = 1;
    while (cs < 8 && blocks * cs < 512 && CiB % (cs * 2) == 0 && CiB / (cs * 2) >= 2) cs *= 2;
    return cs;
}

}  // namespace
}  // namespace st
