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
#include <type_traits>

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
};

// CS = number of wavefronts that share one task, each reducing 1/CS of the input channels; their
// partial tiles are added through LDS at the end (in a fixed order).  CS > 1 multiplies the
// number of wavefronts of a layer with few tiles without shrinking the tile.  A workgroup has
// max(4, CS) wavefronts, each with its own staging region (4.3 KB for 4x8 tiles, 6.8 KB for 8x8):
// up to 108 KB of the 160 KB a gfx950 workgroup may use.
template <int R, int S, int TH, int TW, int KPL, int MINW, int CS, int SD = 1, int SU = 1, int OFF = 0>
__global__ __launch_bounds__(64 * (CS > 4 ? CS : 4), MINW) void fwd_sparse_kernel(Geom g, const float *__restrict__ in,
                                                         const float *__restrict__ f,
                                                         float *__restrict__ out,
                                                         int tiles_w, int tiles_h, int ktiles, int total,
                                                               int slots_per_xcd)
{
    using Cfg = FwdSparseCfg<R, S, TH, TW, KPL, SD, SU, OFF>;
    if (form_deselected(g.sel, g.want, g.thr)) return;          // uniform over the grid, before any barrier
    constexpr int HW = Cfg::HW, HP = Cfg::HP, NXV = Cfg::NXV, PST = Cfg::PST;
    constexpr int WAVES = CS > 4 ? CS : 4;          // wavefronts per workgroup
    __shared__ __attribute__((aligned(16))) float lds_all[WAVES][kBlk * PST];

    // the wavefront index is the same in every lane: kept in a scalar register, and with it every tile coordinate
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;
    const int cpart = wave % CS;                    // which share of the input channels
    // Workgroup -> (tile slot, output-channel tile).  Consecutive workgroup ids are dealt round-robin
    // to the 8 XCDs, each with its own L2; workgroups 8 ids apart run on the same XCD one after the
    // other.  Every XCD gets a contiguous range of pixel tiles and walks it tile by tile, all
    // output-channel tiles of a pixel tile first: the input halo shared by those workgroups, and the
    // halo columns shared with the next pixel tile, are fetched into that L2 once.
    constexpr int TPW = WAVES / CS;                 // tasks (pixel tiles) per workgroup
    const int xcd = blockIdx.x % 8, seq = blockIdx.x / 8;
    const int kt = seq % ktiles;
    const int tile = (xcd * slots_per_xcd + seq / ktiles) * TPW + wave / CS;
    const bool valid = tile < total;                // an invalid wavefront only takes part in barriers
    float *lds = lds_all[wave];

    int t = valid ? tile : 0;
    const int tw = t % tiles_w; t /= tiles_w;
    const int th = t % tiles_h;
    const int n = t / tiles_h;
    const int oh0 = th * TH, ow0 = tw * TW;
    // first input sample of the halo; with SU = 2 the host guarantees that the division is exact
    // (even tile sizes, padding of the same parity as OFF)
    const int ih0 = (oh0 * SD - g.ph + OFF) / SU, iw0 = (ow0 * SD - g.pw + OFF) / SU;
    const int CiB = g.Ci / kBlk, KoB = g.Ko / kBlk;

    float acc[KPL][TH * TW];
#pragma unroll
    for (int j = 0; j < KPL; ++j)
#pragma unroll
        for (int i = 0; i < TH * TW; ++i) acc[j][i] = 0.f;

    // filter pointer of this lane's channel(s) in the wavefront-ordered copy: element [k/64][c][v][u][k%64]
    const float *fp[KPL];
    bool kact[KPL];
#pragma unroll
    for (int j = 0; j < KPL; ++j) {
        const int k = kt * Cfg::KT + j * kWave + lane;
        kact[j] = k < g.Ko;
        // group of 64 channels this lane belongs to; an inactive lane reads element 0 (always written)
        fp[j] = f + (kact[j] ? (size_t)(k / kWave) * g.Ci * (S * R * kWave) + lane : 0);
    }

    // filters of one input channel (flat index c = 16*cb + ci): R*S*KPL registers per lane
    auto load_w = [&](int c, float (&wv)[KPL][S * R]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < KPL; ++j) {
            const float *p = fp[j] + (size_t)c * (S * R * kWave);
#pragma unroll
            for (int tp = 0; tp < S * R; ++tp) wv[j][tp] = p[tp * kWave];
        }
    };

    // all multiply-adds of one input channel of the staged block
    auto process = [&](int ci, const float (&wv)[KPL][S * R]) __attribute__((always_inline)) {
        // Non-zero mask of this channel's halo: one pixel per lane, one compare, one ballot.
        unsigned m32[2 * NXV];
#pragma unroll
        for (int j = 0; j < NXV; ++j) {
            const int pix = j * kWave + lane;
            const float xv = (pix < HP) ? lds[ci * PST + pix] : 0.f;
            const unsigned long long m = __builtin_amdgcn_ballot_w64(xv != 0.f);
            m32[2 * j] = (unsigned)m;
            m32[2 * j + 1] = (unsigned)(m >> 32);
        }
        // The values themselves are read four pixels at a time with one LDS read whose address is
        // the same in every lane (a broadcast): each lane then holds the four inputs in registers
        // and the multiply-adds need no cross-lane move.  The next group is in flight while the
        // current one is processed; LDS reads return in order, so lgkmcnt(1) means "all but the
        // newest read have arrived".  (Staging the filters in LDS, shared by the four wavefronts of
        // a workgroup, was measured and is slower at every sparsity: the barriers cost more than
        // the L2 traffic they save.)
        const float4 *lds4 = reinterpret_cast<const float4 *>(lds + ci * PST);
        constexpr int NG = (HP + 3) / 4;
        float4 xq[2];                       // two groups of values alternate (no register copies)
        xq[0] = lds4[0];
        static_for<0, NG>([&](auto G) __attribute__((always_inline)) {
            constexpr int gidx = decltype(G)::value;
            if constexpr (gidx + 1 < NG) xq[(gidx + 1) % 2] = lds4[gidx + 1];
            // a group whose four pixels are all zero costs one test instead of four, and does not
            // wait for its values either
            constexpr unsigned gmask = 0xFu << ((gidx * 4) % 32);
            if (__builtin_expect((m32[(gidx * 4) / 32] & gmask) != 0u, 1)) {
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
                                for (int j = 0; j < KPL; ++j)
                                    acc[j][ol * TW + oc] = fmaf(xs, wv[j][v * R + u], acc[j][ol * TW + oc]);
                            }
                        }
                    }
                }
            });
            }
        });
    };

    // Two filter register sets alternate: the loads for channel c+1 are in flight while the
    // multiply-adds of channel c run, so the L2 latency of the filter stream is hidden.
    constexpr int NST = (HP * 4 + 63) / 64;         // halo staging slots (pixel, channel quarter) per lane

    const int cb_begin = cpart * (CiB / CS), cb_end = cb_begin + CiB / CS;      // CiB % CS == 0
    const int c_last = cb_end * kBlk - 1;
    float wA[KPL][S * R], wB[KPL][S * R];
    load_w(cb_begin * kBlk, wA);
    // s_waitcnt vmcnt(NW) with the other counters left at their maxima: vector loads return in
    // order, so this waits for everything older than the NW most recent loads (one filter set).
    constexpr int NW = KPL * S * R;
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
#pragma unroll
            for (int jj = 0; jj < NST; ++jj) {
                const int idx = jj * kWave + sl;
                const int pix = idx >> 2, q = idx & 3;
                if (pix < HP) {
                    const int ih = ih0 + pix / HW, iw = iw0 + pix % HW;
                    float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (ih >= 0 && ih < g.Hi && iw >= 0 && iw < g.Wi)
                        val = *reinterpret_cast<const float4 *>(plane + (ih * g.Wi + iw) * kBlk + q * 4);
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

        if constexpr (R * S == 1) {
            // 1x1: a channel step is only TH*TW tests long, so the walk over the alive mask would cost
            // more than it saves; every channel is processed
            for (int ci = 0; ci < kBlk; ci += 2) {
                const int c = cb * kBlk + ci;
                load_w(c + 1, wB);
                __builtin_amdgcn_s_waitcnt(kWaitOlderSet);     // wA has arrived; wB stays in flight
                process(ci, wA);
                load_w(min(c + 2, c_last), wA);
                __builtin_amdgcn_s_waitcnt(kWaitOlderSet);
                process(ci + 1, wB);
            }
            continue;
        }
        // Dead channels cost neither a filter load nor a pass over the masks.  wA holds the filters
        // of channel 0 of this block on entry and of the next block on exit; the filters of the next
        // alive channel are always in flight while the current one is processed.
        const int cnext = min((cb + 1) * kBlk, c_last);      // first channel of the next block
        unsigned bits = __builtin_amdgcn_readfirstlane(alive);      // wave-uniform by construction; say so
        int c0 = bits ? __builtin_ctz(bits) : kBlk;         // kBlk = none (left)
        bits &= bits - 1u;                                  // no-op on 0
        if (c0 != 0) load_w(c0 < kBlk ? cb * kBlk + c0 : cnext, wA);
        while (c0 < kBlk) {
            // the next two alive channels; when none is left the filters of the next block's channel 0
            // are fetched instead, which also keeps the number of loads per step fixed
            const int c1 = bits ? __builtin_ctz(bits) : kBlk;
            bits &= bits - 1u;
            const int c2 = bits ? __builtin_ctz(bits) : kBlk;
            bits &= bits - 1u;
            load_w(c1 < kBlk ? cb * kBlk + c1 : cnext, wB);
            __builtin_amdgcn_s_waitcnt(kWaitOlderSet);     // wA has arrived; wB stays in flight
            process(c0, wA);
            load_w(c2 < kBlk ? cb * kBlk + c2 : cnext, wA);
            __builtin_amdgcn_s_waitcnt(kWaitOlderSet);
            if (c1 < kBlk) process(c1, wB);
            c0 = c2;
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
                        acc[(c0 + i) / (TH * TW)][(c0 + i) % (TH * TW)] += lds_all[wave + pp][i * kWave + lane];
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

template <int R, int S, int TH, int TW, int KPL, int MINW, int CS, int SD, int SU, int OFF>
hipError_t launch_cs(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    using Cfg = FwdSparseCfg<R, S, TH, TW, KPL, SD, SU, OFF>;
    const int tiles_w = ceil_div(g.Wo, TW), tiles_h = ceil_div(g.Ho, TH);
    const int ktiles = ceil_div(g.Ko, Cfg::KT);
    const long long tiles = (long long)tiles_w * tiles_h * g.N;
    constexpr int waves = CS > 4 ? CS : 4;
    constexpr int per_wg = waves / CS;
    const long long slots = (tiles + per_wg - 1) / per_wg;             // workgroups per output-channel tile
    const long long slots_per_xcd = (slots + 7) / 8;
    const long long blocks = slots_per_xcd * 8 * ktiles;
    if (tiles > 0x7fffffffLL || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((fwd_sparse_kernel<R, S, TH, TW, KPL, MINW, CS, SD, SU, OFF>), dim3((unsigned)blocks), dim3(64 * waves), 0, s,
                       g, in, f, out, tiles_w, tiles_h, ktiles, (int)tiles, (int)slots_per_xcd);
    return hipGetLastError();
}

// Picks the channel split: layers with few tiles get 2, 4, 8 or 16 wavefronts per task so that the chip
// (1024 SIMDs x 4 resident wavefronts) is filled and the tail is short: a wavefront walks its share
// of the input channels one after the other, about 1.7 us per channel, so a launch that leaves
// half the wavefront slots empty is as slow as one that fills them.
template <int R, int S, int TH, int TW, int KPL, int MINW, int SD = 1, int SU = 1, int OFF = 0>
hipError_t launch_cfg(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    using Cfg = FwdSparseCfg<R, S, TH, TW, KPL, SD, SU, OFF>;
    const long long tasks = (long long)ceil_div(g.Wo, TW) * ceil_div(g.Ho, TH) * ceil_div(g.Ko, Cfg::KT) * g.N;
    const int CiB = g.Ci / kBlk;
    constexpr bool deep = R == 3 && SD == 1 && SU == 1;     // 8- and 16-way splits: unit-stride 3x3 only
    int cs = 1;
    if (CiB >= 4 && CiB % 2 == 0) cs = 2;
    if ((CiB >= 16 || tasks < 3072) && CiB % 4 == 0) cs = 4;
    if (deep && tasks <= 512 && CiB % 8 == 0) cs = 8;
    if (deep && tasks <= 256 && CiB % 16 == 0) cs = 16;
    if constexpr (deep) {
        if (cs == 16) return launch_cs<R, S, TH, TW, KPL, MINW, 16, SD, SU, OFF>(g, in, f, out, s);
        if (cs == 8) return launch_cs<R, S, TH, TW, KPL, MINW, 8, SD, SU, OFF>(g, in, f, out, s);
    }
    if (cs == 4) return launch_cs<R, S, TH, TW, KPL, MINW, 4, SD, SU, OFF>(g, in, f, out, s);
    if (cs == 2) return launch_cs<R, S, TH, TW, KPL, MINW, 2, SD, SU, OFF>(g, in, f, out, s);
    return launch_cs<R, S, TH, TW, KPL, MINW, 1, SD, SU, OFF>(g, in, f, out, s);
}

}  // namespace

bool fwd_sparse_supported(const Geom &g)
{
    if (g.sw != g.sh || g.uw != g.uh) return false;
    if (g.sw == 2 && g.uw == 1)                     // stride-2 3x3 layers (FWD)
        return g.R == 3 && g.S == 3 && g.pw <= 2 && g.ph <= 2;
    if (g.sw == 1 && g.uw == 2)                     // their BWI: input samples on every second position
        return g.R == 3 && g.S == 3 && g.pw == 1 && g.ph == 1;
    if (g.sw != 1 || g.uw != 1) return false;
    if (g.R == 3 && g.S == 3) return g.pw <= 2 && g.ph <= 2;
    if (g.R == 1 && g.S == 1) return g.pw == 0 && g.ph == 0;
    return false;
}

// Break-even points measured on the layer shapes of the paper's Table 1: the zero-skipping form needs 20-25 % zeros
// with 128 output channels per wavefront and about 60 % with 64; the stride-2 FWD tests 2.25 taps
// per element and its BWI is held by the filter stream of small tiles; a 1x1 layer saves K/64
// multiply-adds per zero.
unsigned fwd_sparse_threshold(const Geom &g)
{
    if (!fwd_sparse_supported(g)) return 0;         // generic kernels: the test only ever removes work
    if (g.R == 1) return g.Ko % 256 == 0 ? 900 : 1001;
    if (g.sw == 2) return 800;
    if (g.uw == 2) return 450;
    const bool wide = g.Ko % 128 == 0;
    return wide ? 250 : 620;
}

namespace {

// Filters in the order the wavefronts read them: wl[Ko/64][Ci][S][R][64 k] for the correlation g the
// kernel runs (Ko rounded up to whole groups of 64; the padding is never written and never used).
// One load instruction of a wavefront then covers 256 contiguous bytes instead of four 64-byte pieces of
// four cache lines, and the nine taps of a channel sit at immediate offsets of one address.  transpose
// selects the BWI form (channel roles exchanged, taps reversed; SparseTrain Sec. 3.3): KB x CB are
// the filter blocks of the LAYER, w its filters in the library layout.
template <bool TRANSPOSE>
__global__ __launch_bounds__(256) void wave_filters_kernel(int KB, int CB, int S, int R,
                                                           const float *__restrict__ w, float *__restrict__ wl,
                                                           const unsigned *sel, unsigned thr)
{
    if (form_deselected(sel, 0, thr)) return;       // the copy of a form that will not run is not written
    __shared__ float tile[kBlk][kBlk + 1];
    int t = blockIdx.x;
    const int u = t % R; t /= R;
    const int v = t % S; t /= S;
    const int cb = t % CB;
    const int kb = t / CB;
    const int a = threadIdx.x / kBlk, b = threadIdx.x % kBlk;
    const size_t src = ((((size_t)kb * CB + cb) * S + v) * R + u) * (kBlk * kBlk);        // [ci = a][ki = b]
    const int SR = S * R;
    if constexpr (!TRANSPOSE) {
        const int k = kb * kBlk + b, c = cb * kBlk + a;
        wl[((size_t)(k / kWave) * (CB * kBlk) + c) * (SR * kWave) + (v * R + u) * kWave + k % kWave] = w[src + a * kBlk + b];
    } else {
        tile[a][b] = w[src + a * kBlk + b];
        __syncthreads();
        // produced channel = c (fast index b), reduced channel = k (a)
        const int c = cb * kBlk + b, k = kb * kBlk + a;
        wl[((size_t)(c / kWave) * (KB * kBlk) + k) * (SR * kWave) + ((S - 1 - v) * R + (R - 1 - u)) * kWave + c % kWave] = tile[b][a];
    }
}

}  // namespace

size_t fwd_sparse_filter_bytes(const Geom &g)
{
    return (size_t)ceil_div(g.Ko, kWave) * kWave * g.Ci * g.S * g.R * sizeof(float);
}

hipError_t launch_wave_filters(const Geom &g, bool transpose, const float *w, float *wl, hipStream_t s)
{
    const int KB = (transpose ? g.Ci : g.Ko) / kBlk, CB = (transpose ? g.Ko : g.Ci) / kBlk;     // of the layer
    const long long blocks = (long long)KB * CB * g.S * g.R;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (transpose)
        hipLaunchKernelGGL(wave_filters_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, KB, CB, g.S, g.R, w, wl, g.sel, g.thr);
    else
        hipLaunchKernelGGL(wave_filters_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, KB, CB, g.S, g.R, w, wl, g.sel, g.thr);
    return hipGetLastError();
}

hipError_t launch_fwd_sparse(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    // 64 accumulators per lane (4x8 pixels x 2 channels, or 8x8 pixels x 1 channel) keep the
    // kernel within 128 registers, i.e. 4 wavefronts per SIMD.
    const bool wide = g.Ko % 128 == 0;
    if (g.sw == 2) {
        // stride 2: a 4x8 output tile is fed by a 9x17 input halo, 2.25 taps per tested element on average
        const bool seven = g.Wo % 8 != 0 && g.Wo % 7 == 0;
        if (wide) return seven ? launch_cfg<3, 3, 4, 7, 2, 4, 2, 1, 0>(g, in, f, out, s) : launch_cfg<3, 3, 4, 8, 2, 4, 2, 1, 0>(g, in, f, out, s);
        return seven ? launch_cfg<3, 3, 4, 7, 1, 4, 2, 1, 0>(g, in, f, out, s) : launch_cfg<3, 3, 4, 8, 1, 4, 2, 1, 0>(g, in, f, out, s);
    }
    if (g.uw == 2) {
        // BWI of a stride-2 layer: every tested element feeds all 9 taps; tiles have even sides so
        // that the position of the input samples within a tile is the same for every tile.  One
        // channel per lane and 64-pixel tiles: a dx tile receives only 2.25 taps per pixel and
        // channel, so the filter registers of a channel must serve as many pixels as possible
        // (two channels per lane on 4x8 tiles measured 20-45 % slower).
        const bool fourteen = g.Wo % 8 != 0 && g.Wo % 14 == 0;
        return fourteen ? launch_cfg<3, 3, 4, 14, 1, 4, 1, 2, 1>(g, in, f, out, s) : launch_cfg<3, 3, 8, 8, 1, 4, 1, 2, 1>(g, in, f, out, s);
    }
    if (g.R == 3 && g.S == 3) {
        // 7-wide tiles when the row length is a multiple of 7 but not of 8 (28, 14): no ragged tiles
        const bool seven = g.Wo % 8 != 0 && g.Wo % 7 == 0;
        if (wide) return seven ? launch_cfg<3, 3, 4, 7, 2, 4>(g, in, f, out, s) : launch_cfg<3, 3, 4, 8, 2, 4>(g, in, f, out, s);
        return seven ? launch_cfg<3, 3, 8, 7, 1, 4>(g, in, f, out, s) : launch_cfg<3, 3, 8, 8, 1, 4>(g, in, f, out, s);
    }
    if (g.R == 1 && g.S == 1) {
        // without spatial reuse a non-zero input feeds only KPL multiply-adds per lane: use as many
        // output channels per lane as the layer has (Sec. 5.2 of the paper: T = Q/V for 1x1)
        if (g.Ko % 256 == 0) return launch_cfg<1, 1, 2, 8, 4, 4>(g, in, f, out, s);
        if (wide) return launch_cfg<1, 1, 8, 8, 2, 2>(g, in, f, out, s);
        return launch_cfg<1, 1, 8, 8, 1, 4>(g, in, f, out, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace st
