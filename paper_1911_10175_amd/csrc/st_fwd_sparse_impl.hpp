// Zero-skipping unit-stride correlation for FWD and (with transposed filters) BWI.
//
// Mapping of the paper's method (SparseTrain Sec. 3.1-3.2) onto a CDNA wavefront:
//  * The vectorised dimension is the output channel (Sec. 3.1): one lane owns KPL output
//    channels, a wavefront owns 64*KPL of them.
//  * The output tile (TH x TW pixels per channel) stays in registers for the whole reduction
//    over input channels and taps, the register-resident output buffer of Sec. 3.2.3 extended
//    from a row segment to a 2-D tile (a wavefront has 64*KPL*TH*TW accumulators, not 30).
//  * The tested operand is one input element shared by every lane.  For one input channel the
//    (TH+S-1) x (TW+R-1) input pixels that reach the tile are held one per lane; a single
//    v_cmp over them yields the 64-bit non-zero mask (the vector compare of Alg. 3, vectorised
//    over pixels instead of channels), and each set bit leads to one lane broadcast plus the up
//    to R*S*KPL multiply-adds of that element (T of Sec. 3.1).  A clear bit is a scalar branch
//    over all of them, taken by the whole wavefront, so no lane ever idles on a zero.
//  * Filters for the current input channel (R*S*KPL values per lane) sit in registers and are
//    reused by every non-zero pixel of the tile; they stream from L2 out of a copy of the filters
//    in wavefront order ([Ko/64][Ci][S][R][64 k], written before every launch), 256 contiguous
//    bytes per load instruction.
#include <cstdio>
#include <type_traits>

#pragma once
#include "st_common.hpp"

namespace st {
namespace {

// SD = stride of the correlation (the output samples every SD-th position), SU = spacing of the
// input samples (SU = 2: the input sits on every second position of the grid the taps slide over,
// which is how the BWI of a stride-2 layer looks: Sec. 3.3 of the paper, dX receives O*P times
// more updates per dY element).  With p(a) = a*SU + OFF the grid position of halo pixel a relative
// to the first position the tile's taps reach, tap v of output row ol reads position ol*SD + v, so
// halo pixel a feeds output row (p(a) - v) / SD for every v that makes this an integer in range.
template <int R, int S, int TH, int TW, int KPL, int SD = 1, int SU = 1, int OFF = 0>
struct FwdSparseCfg {
    static_assert(SD == 1 || SU == 1, "strided and dilated at once is not needed");
    static_assert(OFF < SU, "offset of the first input sample within its spacing");
    static constexpr int HH = ((TH - 1) * SD + S - 1 - OFF) / SU + 1;
    static constexpr int HW = ((TW - 1) * SD + R - 1 - OFF) / SU + 1;
    static constexpr int HP = HH * HW;
    static constexpr int NXV = (HP + 63) / 64;              // registers holding one channel of the halo
    static constexpr int PST = ((HP + 7) / 8) * 8 + 4;      // LDS pixel stride, = 4 (mod 8), >= HP rounded up to 4
    static constexpr int KT = 64 * KPL;                     // output channels per wavefront
    static constexpr int NG = (HP + 3) / 4;                 // groups of four halo pixels

    // Filter row v meets halo row a when the grid row of a lies v below an output row of the tile.
    static constexpr bool row_meets(int a, int v)
    {
        const int t = a * SU + OFF - v;
        return t >= 0 && t % SD == 0 && t / SD < TH;
    }
    static constexpr int first_row(int v)
    {
        for (int a = 0; a < HH; ++a)
            if (row_meets(a, v)) return a;
        return HH;
    }
    static constexpr int last_row(int v)
    {
        int r = -1;
        for (int a = 0; a < HH; ++a)
            if (row_meets(a, v)) r = a;
        return r;
    }
    // group of four halo pixels in which filter row v is first / last needed
    static constexpr int first_group(int v) { return first_row(v) * HW / 4; }
    static constexpr int last_group(int v) { return ((last_row(v) + 1) * HW - 1) / 4; }
    // Filter rows fall out of use in the order 0, 1, ..., and none does before the last one is first
    // needed: the refill loads of a channel are then issued in row order after every wait of that channel.
    static constexpr bool rows_in_order()
    {
        for (int v = 0; v + 1 < S; ++v)
            if (last_group(v) > last_group(v + 1) || first_group(v) > first_group(v + 1)) return false;
        return S == 1 || last_group(0) >= first_group(S - 1);
    }
};

// CS = number of wavefronts that share one task, each reducing 1/CS of the input channels; their
// partial tiles are added through LDS at the end (in a fixed order).  CS > 1 multiplies the
// number of wavefronts of a layer with few tiles without shrinking the tile.  A workgroup has
// max(4, CS) wavefronts, each with its own staging region (2.8 KB for 4x4 tiles, 4.3 KB for 4x8,
// 6.8 KB for 8x8): up to 108 KB of the 160 KB a gfx950 workgroup may use.
//
// Instruction issue is what bounds this kernel: a SIMD issues one wave-wide v_fmac_f32 every 2 cycles
// once two or more wavefronts offer them, and a scalar bit test plus branch adds about 5.5 cycles of
// SIMD time to a pixel whatever the occupancy (measured with 4 wavefronts per SIMD; 17 cycles of the
// wavefront's own time when the branch falls through, 29 when it is taken).  Hence as many multiply-adds
// per tested element as registers and filter traffic allow.  Four channels per lane on 16-pixel tiles
// (36 multiply-adds per interior element) were measured and are no faster than two on 32 pixels: the
// filter registers then serve half as many pixels and the 19 TB/s of filter loads this takes at 50 %
// zeros is more than half of what the L1 caches deliver.
// lds_base: WAVES staging regions of kBlk * PST floats (fwd_sparse_lds_floats), 16-byte aligned.  Every
// thread of the workgroup makes the call (the body contains barriers when CS > 1).
template <int R, int S, int TH, int TW, int KPL, int CS, int SD = 1, int SU = 1, int OFF = 0>
constexpr int fwd_sparse_lds_floats() { return (CS > 4 ? CS : 4) * kBlk * FwdSparseCfg<R, S, TH, TW, KPL, SD, SU, OFF>::PST; }

template <int R, int S, int TH, int TW, int KPL, int CS, int SD = 1, int SU = 1, int OFF = 0>
__device__ __forceinline__ void fwd_sparse_body(const Geom &g, const float *__restrict__ in, const float *__restrict__ f,
                                                float *__restrict__ out, int tiles_w, int tiles_h, int ktiles, int total,
                                                int slots_per_xcd, int kt_major, float *lds_base)
{
    using Cfg = FwdSparseCfg<R, S, TH, TW, KPL, SD, SU, OFF>;
    constexpr int HW = Cfg::HW, HP = Cfg::HP, NXV = Cfg::NXV, PST = Cfg::PST, NG = Cfg::NG;
    constexpr int WAVES = CS > 4 ? CS : 4;          // wavefronts per workgroup
    // One filter register set, refilled row by row, for the one-channel-per-lane shapes: it brings them
    // from 120 to under 96 registers, i.e. from 4 to 5 wavefronts per SIMD (measured -8 % time at 50 %
    // zeros).  The unit-stride 3x3 shapes with two channels per lane (PAIRED, below) use it as well: measured
    // against two sets in turn it takes 5-6 % off the 28x28 layers with 512 channels at 50 % zeros and is
    // even elsewhere.  The other shapes keep two sets in turn (the freed registers change no occupancy step
    // there and the shorter prefetch distance costs 5 % at 90 % zeros).
    constexpr bool PAIRED = fwd_sparse_paired(R, S, KPL, SD, SU);
    constexpr bool ROLL = S > 1 && (KPL == 1 || PAIRED);
    constexpr int LPR = PAIRED ? R : KPL * R;       // load instructions per filter row
    constexpr bool WALK = S > 1;                    // dead channels are skipped (3x3 only)
    // Operand order of the multiply-adds written by hand for one channel per lane: with the tested value
    // as first source operand of nine consecutive v_fmac_f32 (the order the compiler picks) the vector
    // pipe issues them 25 % below its rate (measured on the kernel's own register sequence: 107 against
    // 141 TFLOP/s); as second operand it does not (-9 % kernel time).  With two channels per lane the
    // compiler's order is the faster one.
    constexpr bool FMA_BY_HAND = KPL == 1;
    static_assert(!ROLL || Cfg::rows_in_order(), "the waits on the refilled filter rows assume this order");

    // the wavefront index is the same in every lane: kept in a scalar register, and with it every tile coordinate
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;
    const int cpart = wave % CS;                    // which share of the input channels
    // Workgroup -> (tile slot, output-channel tile).  Consecutive workgroup ids are dealt round-robin
    // to the 8 XCDs, each with its own 4 MB L2; workgroups 8 ids apart run on the same XCD one after the
    // other.  Every XCD gets a contiguous range of pixel tiles.  With a small filter tensor it walks the
    // range tile by tile, all output-channel tiles of a pixel tile first: the input halo shared by those
    // workgroups, and the halo columns shared with the next pixel tile, are fetched into that L2 once.
    // With filters that would not stay in L2 next to it (kt_major) it walks the whole range once per
    // output-channel tile instead, so that only one tile's filters (C*S*R*64*KPL values) are live at a
    // time and the input is what is fetched again (measured on 512->512 @28, N = 32: 885 MB -> 328 MB fetched per launch, same time).
    constexpr int TPW = WAVES / CS;                 // tasks (pixel tiles) per workgroup
    const int xcd = blockIdx.x % 8, seq = blockIdx.x / 8;
    const int kt = kt_major ? seq / slots_per_xcd : seq % ktiles;
    const int slot = kt_major ? seq % slots_per_xcd : seq / ktiles;
    const int tile = (xcd * slots_per_xcd + slot) * TPW + wave / CS;
    const bool valid = tile < total;                // an invalid wavefront only takes part in barriers
    float *lds = lds_base + wave * (kBlk * PST);

    int t = valid ? tile : 0;
    const int tw = t % tiles_w; t /= tiles_w;
    const int th = t % tiles_h;
    const int n = t / tiles_h;
    const int oh0 = th * TH, ow0 = tw * TW;
    // first input sample of the halo; with SU = 2 the host guarantees that the division is exact
    // (even tile sizes, padding of the same parity as OFF)
    const int ih0 = (oh0 * SD - g.ph + OFF) / SU, iw0 = (ow0 * SD - g.pw + OFF) / SU;
    const int CiB = g.Ci / kBlk, KoB = g.Ko / kBlk;

    // Register parity.  A wave-wide fp32 multiply-add whose three register operands (accumulator and both
    // factors) all have even or all have odd register numbers issues at half rate in a bare instruction
    // stream (69 against 138 TFLOP/s; any other combination of the 64 is free).  With registers handed out
    // without regard to that, a quarter of the multiply-adds of this kernel are of that kind.  PAIRED (two
    // channels per lane, unit-stride 3x3: the shapes that carry most of the time) rules it out by construction: the two
    // accumulators of a pixel are kept in one 64-bit register pair (process() sees to it), which the hardware
    // requires to start at an even register, channel 1 in its even half and channel 0 in its odd half; the two filter values of a tap
    // arrive by one 8-byte load into another such pair, channel 0 in the even half, channel 1 in the odd half.
    // Accumulator and filter value of a multiply-add then never share a parity, whatever register the tested
    // input value sits in, and a channel's filters take 9 load instructions instead of 18.  Measured on the
    // VGG16 layers at N = 32: 1.5-3 % less time at 0-70 % zeros on top of what the single filter set brings,
    // i.e. far less than the bare streams suggest (between the tests, reads and branches of this kernel the
    // slow multiply-adds mostly find the pipe idle anyway), and 6-7 % MORE at 90 % zeros, where the time goes
    // to the filter stream and the 8-byte loads turn out slower than twice as many 4-byte ones.
    typedef float f2 __attribute__((ext_vector_type(2)));
    float acc[KPL][TH * TW];
#pragma unroll
    for (int j = 0; j < KPL; ++j)
#pragma unroll
        for (int i = 0; i < TH * TW; ++i) acc[j][i] = 0.f;

    // Filters of this wavefront in the wavefront-ordered copy: element [k/64][c][v][u][k%64] with
    // k/64 = kt*KPL + j.  The address is a base that is the same in every lane (scalar registers) plus
    // the lane's own 32-bit offset, so that one vector register serves all loads; a lane beyond Ko reads
    // the unwritten padding of the copy (in bounds, never stored).
    // (PAIRED: element [k/128][c][v][u][k%64][(k/64)%2], the lane's two channels side by side.)
    const float *fw = f + (size_t)kt * KPL * g.Ci * (S * R * kWave);
    const size_t jstride = (size_t)g.Ci * (S * R * kWave);
    const unsigned lane_u = lane;
    // a filter register set: [channel of the lane][tap], or PAIRED [tap] pairs with element j = channel j
    using WSet = std::conditional_t<PAIRED, f2[S * R], float[KPL][S * R]>;

    // filters of filter row v (all rows when v < 0, row by row: the order the waits in process() count
    // on) of input channel c (flat index c = 16*cb + ci)
    auto load_w = [&](int c, WSet &wv, auto V) __attribute__((always_inline)) {
        constexpr int v = decltype(V)::value;
#pragma unroll
        for (int vv = (v < 0 ? 0 : v); vv < (v < 0 ? S : v + 1); ++vv) {
            if constexpr (PAIRED) {
                const f2 *p = reinterpret_cast<const f2 *>(fw + (size_t)c * (S * R * kWave * 2));     // uniform
#pragma unroll
                for (int u = 0; u < R; ++u) wv[vv * R + u] = p[(vv * R + u) * kWave + lane_u];
            } else {
#pragma unroll
                for (int j = 0; j < KPL; ++j) {
                    const float *p = fw + j * jstride + (size_t)c * (S * R * kWave);       // uniform
#pragma unroll
                    for (int u = 0; u < R; ++u) wv[j][vv * R + u] = p[(vv * R + u) * kWave + lane_u];
                }
            }
            // keeps the compiler from regrouping the loads by address across rows
            if (S > 1 && v < 0) __builtin_amdgcn_sched_barrier(0);
        }
    };
    using All = std::integral_constant<int, -1>;

    // All multiply-adds of one input channel of the staged block.  GT = with a test per group of four
    // halo pixels (pays when most groups are all zero).  With ROLL the filter registers of a row are
    // refilled with those of channel cnext as soon as the last halo row that uses them is done.
    // Non-zero mask of one channel's halo: one pixel per lane, one compare, one ballot (the vector
    // compare of Alg. 3 of the paper, over pixels instead of channels).  Returns the number of non-zeros.
    auto halo_mask = [&](int ci, unsigned (&m32)[2 * NXV]) __attribute__((always_inline)) {
        int count = 0;
#pragma unroll
        for (int j = 0; j < NXV; ++j) {
            const int pix = j * kWave + lane;
            const float xv = (pix < HP) ? lds[ci * PST + pix] : 0.f;
            const unsigned long long m = __builtin_amdgcn_ballot_w64(xv != 0.f);
            m32[2 * j] = (unsigned)m;
            m32[2 * j + 1] = (unsigned)(m >> 32);
            count += __builtin_popcountll(m);
        }
        return count;
    };

    auto process = [&](int ci, const unsigned (&m32)[2 * NXV], WSet &wv, int cnext, auto GTc) __attribute__((always_inline)) {
        constexpr bool GT = decltype(GTc)::value;
        // once per channel the two accumulators of a pixel pass through an empty statement as ONE 64-bit
        // operand (channel 1 first): the register allocator then keeps them in an aligned pair throughout
        if constexpr (PAIRED) {
#pragma unroll
            for (int i = 0; i < TH * TW; ++i) {
                f2 t = {acc[1][i], acc[0][i]};
                asm volatile("" : "+v"(t));
                acc[1][i] = t.x;
                acc[0][i] = t.y;
            }
        }

        // The values themselves are read four pixels at a time with one LDS read whose address is
        // the same in every lane (a broadcast): each lane then holds the four inputs in registers
        // and the multiply-adds need no cross-lane move.  The next group is in flight while the
        // current one is processed; LDS reads return in order, so lgkmcnt(1) means "all but the
        // newest read have arrived".
        const float4 *lds4 = reinterpret_cast<const float4 *>(lds + ci * PST);
        float4 xq[2];                       // two groups of values alternate (no register copies)
        xq[0] = lds4[0];
        static_for<0, NG>([&](auto G) __attribute__((always_inline)) {
            constexpr int gidx = decltype(G)::value;
            if constexpr (gidx + 1 < NG) xq[(gidx + 1) % 2] = lds4[gidx + 1];
            // The filter rows first needed in this group were fetched while the previous channel was
            // processed, row v before row v+1; vector loads return in order, so they have arrived once no
            // more loads are outstanding than were issued after them.
            if constexpr (ROLL) {
                static_for<0, S>([&](auto V) __attribute__((always_inline)) {
                    constexpr int v = decltype(V)::value;
                    if constexpr (Cfg::first_group(v) == gidx) __builtin_amdgcn_s_waitcnt(vmcnt_imm(LPR * (S - 1 - v)));
                });
            }
            constexpr unsigned gmask = 0xFu << ((gidx * 4) % 32);
            // with GT a group whose four pixels are all zero costs one test instead of four, and does
            // not wait for its values either
            if (!GT || __builtin_expect((m32[(gidx * 4) / 32] & gmask) != 0u, 1)) {
            if constexpr (gidx + 1 < NG) {
                __builtin_amdgcn_s_waitcnt(0xC17F);      // lgkmcnt(1)
            } else {
                __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0)
            }
            const float4 cur = xq[gidx % 2];
            const float xg[4] = {cur.x, cur.y, cur.z, cur.w};
            // one branch per halo pixel; all register indices below are compile-time constants
            static_for<0, 4>([&](auto J) __attribute__((always_inline)) {
                constexpr int i = gidx * 4 + decltype(J)::value;
                if constexpr (i < HP) {
                    constexpr int a = (i / HW) * SU + OFF, b = (i % HW) * SU + OFF;    // grid position
                    if (__builtin_expect((m32[i / 32] & (1u << (i % 32))) != 0u, 1)) {
                        const float xs = xg[i % 4];
#pragma unroll
                        for (int v = 0; v < S; ++v) {
                            if (a - v < 0 || (a - v) % SD != 0 || (a - v) / SD >= TH) continue;
                            const int ol = (a - v) / SD;
#pragma unroll
                            for (int u = 0; u < R; ++u) {
                                if (b - u < 0 || (b - u) % SD != 0 || (b - u) / SD >= TW) continue;
                                const int oc = (b - u) / SD;
#pragma unroll
                                for (int j = 0; j < KPL; ++j) {
                                    float &a_ref = acc[j][ol * TW + oc];
                                    // PAIRED: channel 0 = odd accumulator and even filter register, channel 1 the reverse
                                    float w_val;
                                    if constexpr (PAIRED) w_val = wv[v * R + u][j];
                                    else w_val = wv[j][v * R + u];
                                    if constexpr (FMA_BY_HAND)
                                        asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(a_ref) : "v"(w_val), "v"(xs));
                                    else
                                        a_ref = fmaf(xs, w_val, a_ref);
                                }
                            }
                        }
                    }
                }
            });
            }
            // filter rows whose last halo row ends in this group: their registers are free, fetch the
            // next channel's values into them
            if constexpr (ROLL) {
                static_for<0, S>([&](auto V) __attribute__((always_inline)) {
                    if constexpr (Cfg::last_group(decltype(V)::value) == gidx) {
                        // the loads stay here: hoisted above the multiply-adds that still read the old
                        // values they would need registers of their own
                        __builtin_amdgcn_sched_barrier(0);
                        load_w(cnext, wv, V);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                });
            }
        });
    };
    // The test per group of four pixels pays from about 70 % zeros (one test instead of four for an
    // all-zero group) and costs three scalar instructions per group, 3-5 % of the time, at 50 %; it is
    // kept in every shape.  (Both forms in one kernel, chosen per channel from the mask's population
    // count, made the compiler spill 90 registers.)
    using WithGroupTest = std::integral_constant<bool, true>;
    using GroupTest = WithGroupTest;

    constexpr int NST = (HP * 4 + 63) / 64;         // halo staging slots (pixel, channel quarter) per lane

    const int cb_begin = cpart * (CiB / CS), cb_end = cb_begin + CiB / CS;      // CiB % CS == 0
    const int c_last = cb_end * kBlk - 1;
    WSet wA;
    std::conditional_t<ROLL, float[1][1], WSet> wB;     // second set: only without the row-by-row refill
    if constexpr (!ROLL) load_w(cb_begin * kBlk, wA, All{});
    // s_waitcnt vmcnt(NW) with the other counters left at their maxima: vector loads return in
    // order, so this waits for everything older than the NW most recent loads (one filter set).
    constexpr int NW = PAIRED ? S * R : KPL * S * R;    // load instructions of one filter set
    static_assert(NW < 64, "vmcnt is a 6-bit counter");
    constexpr int kWaitOlderSet = vmcnt_imm(NW);

    unsigned alive = 0u;
    for (int cb = valid ? cb_begin : cb_end; cb < cb_end; ++cb) {
        // ---- stage the halo of this 16-channel block in LDS, transposed to [channel][pixel] ----
        __builtin_amdgcn_wave_barrier();
        {
            // The slot arithmetic is redone for every block from a lane index the compiler cannot
            // see through: a few dozen instructions per 16 channels, instead of address registers
            // that would stay live (and spill) across the whole reduction.
            int sl = lane;
            asm volatile("" : "+v"(sl));
            const float *plane = in + act_off(n, cb, 0, 0, CiB, g.Hi, g.Wi);      // wave-uniform base
            unsigned nz0 = 0u, nz1 = 0u, nz2 = 0u, nz3 = 0u;    // OR of the value bits per staged component of this lane
            // NB of a lane's 16-byte pieces are asked for before the first of them is written to LDS.  One at a
            // time (load, wait, write) makes NST memory round trips per block of 16 channels; all at once makes
            // one but holds 4 * NST more registers at this point, the kernel's fullest.  The 4x8 tiles with two
            // channels per lane have four wavefronts per SIMD either way and gain 1-2 % at 50 % zeros, 2-4 % at
            // 90 %, the 1x1 shapes 2-5 %; the other 3x3 shapes would fall from five wavefronts to four and
            // lose 5-11 %.
            constexpr int NB = ((PAIRED && TW == 8) || R * S == 1) ? NST : 1;
#pragma unroll
            for (int j0 = 0; j0 < NST; j0 += NB) {
                float4 sv[NB];
#pragma unroll
                for (int jb = 0; jb < NB; ++jb) {
                    const int idx = (j0 + jb) * kWave + sl;
                    const int pix = idx >> 2, q = idx & 3;
                    const int ih = ih0 + pix / HW, iw = iw0 + pix % HW;
                    sv[jb] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (j0 + jb < NST && pix < HP && ih >= 0 && ih < g.Hi && iw >= 0 && iw < g.Wi)
                        sv[jb] = *reinterpret_cast<const float4 *>(plane + (ih * g.Wi + iw) * kBlk + q * 4);
                }
#pragma unroll
                for (int jb = 0; jb < NB; ++jb) {
                    const int idx = (j0 + jb) * kWave + sl;
                    const int pix = idx >> 2, q = idx & 3;
                    if (j0 + jb < NST && pix < HP) {
                        const float4 val = sv[jb];
                        lds[(q * 4 + 0) * PST + pix] = val.x;
                        lds[(q * 4 + 1) * PST + pix] = val.y;
                        lds[(q * 4 + 2) * PST + pix] = val.z;
                        lds[(q * 4 + 3) * PST + pix] = val.w;
                        if constexpr (R * S != 1) {
                            nz0 |= __builtin_bit_cast(unsigned, val.x);
                            nz1 |= __builtin_bit_cast(unsigned, val.y);
                            nz2 |= __builtin_bit_cast(unsigned, val.z);
                            nz3 |= __builtin_bit_cast(unsigned, val.w);
                        }
                    }
                }
            }
            // Channels of this block with at least one non-zero in the halo (ReLU leaves whole
            // channels of an image dead): a lane's slots all belong to channel quarter lane % 4
            // (64 % 4 == 0), so channel 4*q + comp is alive iff some lane = q (mod 4) saw a
            // non-zero in component comp.  -0 counts as zero, denormals do not.
            alive = 0u;
            const unsigned nzv[4] = {nz0, nz1, nz2, nz3};
#pragma unroll
            for (int comp = 0; comp < (R * S != 1 ? 4 : 0); ++comp) {
                const unsigned long long m = __builtin_amdgcn_ballot_w64((nzv[comp] & 0x7fffffffu) != 0u);
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (m & (0x1111111111111111ull << q)) alive |= 1u << (q * 4 + comp);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        if constexpr (!WALK) {
            // 1x1: a channel step is only TH*TW tests long, so the walk over the alive mask would cost
            // more than it saves; every channel is processed, with two filter register sets in turn
            for (int ci = 0; ci < kBlk; ci += 2) {
                const int c = cb * kBlk + ci;
                unsigned m32[2 * NXV];
                load_w(c + 1, wB, All{});
                __builtin_amdgcn_s_waitcnt(kWaitOlderSet);     // wA has arrived; wB stays in flight
                halo_mask(ci, m32);
                process(ci, m32, wA, 0, WithGroupTest{});
                load_w(min(c + 2, c_last), wA, All{});
                __builtin_amdgcn_s_waitcnt(kWaitOlderSet);
                halo_mask(ci + 1, m32);
                process(ci + 1, m32, wB, 0, WithGroupTest{});
            }
        } else if constexpr (!ROLL) {
            // two filter register sets in turn, the filters of the next alive channel always in flight
            const int cnext = min((cb + 1) * kBlk, c_last);      // first channel of the next block
            unsigned bits = __builtin_amdgcn_readfirstlane(alive);
            int c0 = bits ? __builtin_ctz(bits) : kBlk;
            bits &= bits - 1u;
            if (c0 != 0) load_w(c0 < kBlk ? cb * kBlk + c0 : cnext, wA, All{});
            while (c0 < kBlk) {
                const int c1 = bits ? __builtin_ctz(bits) : kBlk;
                bits &= bits - 1u;
                const int c2 = bits ? __builtin_ctz(bits) : kBlk;
                bits &= bits - 1u;
                unsigned m32[2 * NXV];
                load_w(c1 < kBlk ? cb * kBlk + c1 : cnext, wB, All{});
                __builtin_amdgcn_s_waitcnt(kWaitOlderSet);     // wA has arrived; wB stays in flight
                halo_mask(c0, m32);
                process(c0, m32, wA, 0, GroupTest{});
                load_w(c2 < kBlk ? cb * kBlk + c2 : cnext, wA, All{});
                __builtin_amdgcn_s_waitcnt(kWaitOlderSet);
                if (c1 < kBlk) {
                    halo_mask(c1, m32);
                    process(c1, m32, wB, 0, GroupTest{});
                }
                c0 = c2;
            }
        } else {
            // Dead channels cost neither a filter load nor a pass over the masks.  wA holds (or is
            // receiving) the filters of channel 0 of this block on entry and of the next block on exit.
            const int cnext = min((cb + 1) * kBlk, c_last);      // first channel of the next block
            unsigned bits = __builtin_amdgcn_readfirstlane(alive);      // wave-uniform by construction; say so
            int c0 = bits ? __builtin_ctz(bits) : kBlk;         // kBlk = none (left)
            bits &= bits - 1u;                                  // no-op on 0
            // (the first block fetches its first set here, not ahead of the loop: every full fetch is then
            // issued row by row from this one place, which is what the compiler's own wait counting needs
            // to agree with the waits in process())
            if (c0 != 0 || cb == cb_begin) load_w(c0 < kBlk ? cb * kBlk + c0 : cnext, wA, All{});
            while (c0 < kBlk) {
                const int c1 = bits ? __builtin_ctz(bits) : kBlk;
                bits &= bits - 1u;
                const int cn = c1 < kBlk ? cb * kBlk + c1 : cnext;
                // zero fraction of this channel's halo decides which form of the pixel loop runs: the
                // group test pays from about 70 % zeros
                unsigned m32[2 * NXV];
                halo_mask(c0, m32);
                process(c0, m32, wA, cn, GroupTest{});
                c0 = c1;
            }
        }
    }

    // ---- add the partial tiles of the CS wavefronts of a task (fixed order: share 0 + 1 + ...) ----
    if constexpr (CS > 1) {
        constexpr int NACC = KPL * TH * TW;
        constexpr int CHUNK = (NACC % 8 == 0 && 8 * kWave <= kBlk * PST) ? 8 : (NACC % 4 == 0 && 4 * kWave <= kBlk * PST) ? 4 : 1;
        static_assert(NACC % CHUNK == 0 && CHUNK * kWave <= kBlk * PST, "reduction chunk must fit the staging region");
#pragma unroll
        for (int c0 = 0; c0 < NACC; c0 += CHUNK) {
            __syncthreads();                        // the staging region / previous chunk is no longer read
            if (cpart != 0) {
#pragma unroll
                for (int i = 0; i < CHUNK; ++i) lds[i * kWave + lane] = acc[(c0 + i) / (TH * TW)][(c0 + i) % (TH * TW)];
            }
            __syncthreads();
            if (cpart == 0) {
#pragma unroll
                for (int pp = 1; pp < CS; ++pp)
#pragma unroll
                    for (int i = 0; i < CHUNK; ++i)
                        acc[(c0 + i) / (TH * TW)][(c0 + i) % (TH * TW)] += lds_base[(wave + pp) * (kBlk * PST) + i * kWave + lane];
            }
        }
    }

    // ---- store the tile ----
    // The lane index is passed through an empty asm so that the compiler cannot hoist the store
    // address arithmetic above the main loop, where it would be spilled to scratch for the whole
    // reduction (the kernel runs at the 128-register limit of 4 wavefronts per SIMD).
    int lane_late = lane;
    asm volatile("" : "+v"(lane_late));
    if (valid && cpart == 0) {
#pragma unroll
        for (int j = 0; j < KPL; ++j) {
            const int k = kt * Cfg::KT + j * kWave + lane_late;
            if (k >= g.Ko) continue;
            const int kb = k / kBlk, ki = k % kBlk;
            float *op = out + act_off(n, kb, oh0, ow0, KoB, g.Ho, g.Wo) + ki;
#pragma unroll
            for (int a = 0; a < TH; ++a) {
                if (oh0 + a >= g.Ho) continue;
#pragma unroll
                for (int b = 0; b < TW; ++b) {
                    if (ow0 + b >= g.Wo) continue;
                    op[(a * g.Wo + b) * kBlk] = acc[j][a * TW + b];
                }
            }
        }
    }
}

template <int R, int S, int TH, int TW, int KPL, int MINW, int CS, int SD = 1, int SU = 1, int OFF = 0>
__global__ __launch_bounds__(64 * (CS > 4 ? CS : 4), MINW) void fwd_sparse_kernel(Geom g, const float *__restrict__ in,
                                                                                  const float *__restrict__ f,
                                                                                  float *__restrict__ out, int tiles_w,
                                                                                  int tiles_h, int ktiles, int total,
                                                                                  int slots_per_xcd, int kt_major)
{
    if (form_deselected(g.sel, g.want, g.thr)) return;          // uniform over the grid, before any barrier
    __shared__ __attribute__((aligned(16))) float lds_all[fwd_sparse_lds_floats<R, S, TH, TW, KPL, CS, SD, SU, OFF>()];
    fwd_sparse_body<R, S, TH, TW, KPL, CS, SD, SU, OFF>(g, in, f, out, tiles_w, tiles_h, ktiles, total, slots_per_xcd, kt_major,
                                                        lds_all);
}

// Grid of a launch with CS wavefronts per task
struct SparseGrid {
    int tiles_w, tiles_h, ktiles, total, slots_per_xcd, kt_major;
    long long blocks;
    bool ok;
};

template <int TH, int TW, int KT, int CS>
SparseGrid sparse_grid(const Geom &g)
{
    SparseGrid q;
    q.tiles_w = ceil_div(g.Wo, TW);
    q.tiles_h = ceil_div(g.Ho, TH);
    q.ktiles = ceil_div(g.Ko, KT);
    const long long tiles = (long long)q.tiles_w * q.tiles_h * g.N;
    constexpr int waves = CS > 4 ? CS : 4;
    constexpr int per_wg = waves / CS;
    const long long slots = (tiles + per_wg - 1) / per_wg;             // workgroups per output-channel tile
    const long long slots_per_xcd = (slots + 7) / 8;
    q.blocks = slots_per_xcd * 8 * q.ktiles;
    q.ok = tiles <= 0x7fffffffLL && q.blocks <= 0x7fffffffLL;
    q.total = (int)tiles;
    q.slots_per_xcd = (int)slots_per_xcd;
    // all filters of the layer against the 4 MB of one XCD's L2, which the input stream needs part of
    q.kt_major = q.ktiles > 1 && fwd_sparse_filter_bytes(g) > kFilterBytesTileMajor;
    return q;
}

template <int R, int S, int TH, int TW, int KPL, int MINW, int CS, int SD, int SU, int OFF>
hipError_t launch_cs(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    using Cfg = FwdSparseCfg<R, S, TH, TW, KPL, SD, SU, OFF>;
    const SparseGrid q = sparse_grid<TH, TW, Cfg::KT, CS>(g);
    if (!q.ok) return hipErrorInvalidValue;
    constexpr int waves = CS > 4 ? CS : 4;
    if (g.describe) {
        snprintf(g.describe, (size_t)g.describe_len, "fwd_sparse_kernel<%d, %d, %d, %d, %d, %d, %d, %d, %d, %d>", R, S, TH, TW, KPL,
                 MINW, CS, SD, SU, OFF);
        return hipSuccess;
    }
    hipLaunchKernelGGL((fwd_sparse_kernel<R, S, TH, TW, KPL, MINW, CS, SD, SU, OFF>), dim3((unsigned)q.blocks), dim3(64 * waves), 0, s,
                       g, in, f, out, q.tiles_w, q.tiles_h, q.ktiles, q.total, q.slots_per_xcd, q.kt_major);
    return hipGetLastError();
}

// Picks the channel split: layers with few tiles get 2, 4, 8 or 16 wavefronts per task so that the chip
// (1024 SIMDs x 4 resident wavefronts) is filled and the tail is short: a wavefront walks its share
// of the input channels one after the other, about 1.7 us per channel, so a launch that leaves
// half the wavefront slots empty is as slow as one that fills them.  deep = 8- and 16-way splits allowed
// (unit-stride 3x3 only).
inline int sparse_channel_split(const Geom &g, int TH, int TW, int KT, bool deep)
{
    const long long tasks = (long long)ceil_div(g.Wo, TW) * ceil_div(g.Ho, TH) * ceil_div(g.Ko, KT) * g.N;
    const int CiB = g.Ci / kBlk;
    int cs = 1;
    if (CiB >= 4 && CiB % 2 == 0) cs = 2;
    if ((CiB >= 16 || tasks < 3072) && CiB % 4 == 0) cs = 4;
    if (deep && tasks <= 512 && CiB % 8 == 0) cs = 8;
    if (deep && tasks <= 256 && CiB % 16 == 0) cs = 16;
    return cs;
}

template <int R, int S, int TH, int TW, int KPL, int MINW, int SD = 1, int SU = 1, int OFF = 0>
hipError_t launch_cfg(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    using Cfg = FwdSparseCfg<R, S, TH, TW, KPL, SD, SU, OFF>;
    constexpr bool deep = R == 3 && SD == 1 && SU == 1;
    const int cs = sparse_channel_split(g, TH, TW, Cfg::KT, deep);
    if constexpr (deep) {
        if (cs == 16) return launch_cs<R, S, TH, TW, KPL, MINW, 16, SD, SU, OFF>(g, in, f, out, s);
        if (cs == 8) return launch_cs<R, S, TH, TW, KPL, MINW, 8, SD, SU, OFF>(g, in, f, out, s);
    }
    if (cs == 4) return launch_cs<R, S, TH, TW, KPL, MINW, 4, SD, SU, OFF>(g, in, f, out, s);
    if (cs == 2) return launch_cs<R, S, TH, TW, KPL, MINW, 2, SD, SU, OFF>(g, in, f, out, s);
    return launch_cs<R, S, TH, TW, KPL, MINW, 1, SD, SU, OFF>(g, in, f, out, s);
}

}  // namespace
}  // namespace st
