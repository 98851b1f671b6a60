// Dense 1x1 (pointwise) unit-stride correlation on the matrix cores: the dense control of the
// 1x1 layers (SparseTrain Table 1, the resnet*_1*, *_3 rows), used for FWD and, with transposed
// filters, for BWI.
//
// A 1x1 layer is a plain matrix product per pixel (Sec. 5.2 of the paper makes the same remark):
// out[k][pixel] = sum_c f[k][c] * in[c][pixel] over all N*H*W pixels.  There is no halo and no
// reuse of an input element between pixels, so nothing is staged in LDS and there are no
// barriers: with v_mfma_f32_32x32x2_f32 (rows = 32 output channels, columns = 32 pixels,
// reduction = 2 input channels) a lane supplies, for its pixel, 8 of the 16 channels of a block,
// which are 32 contiguous bytes of the blocked activation layout, i.e. the operand is loaded
// from global memory in the order the instruction consumes it.  The filter operand comes from
// the reformatted copy the 3x3 dense kernel uses, [K/32][C/16][c half][32 k][8 c].
//
// These layers sit at or below the ridge of the roofline (25 flop/B for 256 -> 64 channels), so
// the kernel is built to keep many bytes in flight: each wavefront owns PB*32 pixels and KB*32
// output channels and keeps the input of the next DEPTH-1 channel blocks and the filters of the
// next block in registers while the MFMAs of the current block run.  Pixels are numbered across
// the whole minibatch (n*H*W + p), so image sizes that are no multiple of the tile (28x28,
// 14x14, 7x7) leave no ragged tiles except the very last one.
#include <cstdlib>
#include <type_traits>

#include "st_common.hpp"

namespace st {
namespace {

template <int PB, int KB, int DEPTH>
__global__ __launch_bounds__(256) void pw_dense_kernel(int total_px, int HW, int CiB, int KoB,
                                                       const float *__restrict__ in,
                                                       const float *__restrict__ wd,
                                                       float *__restrict__ out, int kgroups,
                                                       const unsigned *sel, unsigned thr)
{
    if (form_deselected(sel, 1, thr)) return;
    // the wavefront index is the same in every lane: kept in a scalar register, and with it every tile coordinate
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;
    const int l32 = lane % 32, half = lane / 32;
    // workgroup id -> (pixel group, channel group): the channel groups of one pixel group get ids that
    // are equal modulo 8, i.e. run on the same XCD, and share the input through that XCD's L2
    const int kg = (blockIdx.x / 8) % kgroups;
    const int pg = (blockIdx.x / (8 * kgroups)) * 8 + blockIdx.x % 8;
    const long long px0 = ((long long)pg * 4 + wave) * (32 * PB);
    if (px0 >= total_px) return;                    // whole wavefront past the end (no barriers in this kernel)

    // this lane's pixel of each 32-pixel block; lanes past the end read the last pixel and store nothing
    size_t ibase[PB], obase[PB];
    bool pvalid[PB];
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
        int gp = (int)px0 + pb * 32 + l32;          // px0 < total_px, and the host keeps total_px + 64 in int range
        pvalid[pb] = gp < total_px;
        if (!pvalid[pb]) gp = total_px - 1;
        const int n = gp / HW, p = gp % HW;
        ibase[pb] = ((size_t)n * CiB * HW + p) * kBlk + half * 8;
        obase[pb] = ((size_t)n * KoB * HW + p) * kBlk;
    }
    const size_t plane = (size_t)HW * kBlk;

    floatx16 acc[KB][PB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[kb][pb][r] = 0.f;

    // filter operand: lane supplies f[k = (kg*KB + kb)*32 + l32][c = cb*16 + half*8 + j], j = 0..7
    const float *wbase = wd + (size_t)kg * KB * CiB * 512 + half * 256 + l32 * 8;

    float4 xr[DEPTH][PB][2];
    float4 wr[DEPTH][KB][2];
    auto load_x = [&](int cb, float4 (&dst)[PB][2]) __attribute__((always_inline)) {
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            const float4 *p = reinterpret_cast<const float4 *>(in + ibase[pb] + (size_t)cb * plane);
            dst[pb][0] = p[0];
            dst[pb][1] = p[1];
        }
    };
    auto load_w = [&](int cb, float4 (&dst)[KB][2]) __attribute__((always_inline)) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const float4 *p = reinterpret_cast<const float4 *>(wbase + ((size_t)kb * CiB + cb) * 512);
            dst[kb][0] = p[0];
            dst[kb][1] = p[1];
        }
    };

    // prologue: blocks 0 .. DEPTH-2 (indices clamped: a short channel loop re-reads its last block,
    // which keeps the number of loads issued per step fixed)
    static_for<0, DEPTH - 1>([&](auto J) __attribute__((always_inline)) {
        constexpr int j = decltype(J)::value;
        load_w(min(j, CiB - 1), wr[j]);
        load_x(min(j, CiB - 1), xr[j]);
    });

    // Step cb requests block cb+DEPTH-1 and then needs block cb, requested DEPTH-1 steps earlier:
    // loads return in order, so "all but the newest (DEPTH-1) * (2*KB + 2*PB)" is exactly that.
    constexpr int kWaitOlder = vmcnt_imm((DEPTH - 1) * (2 * PB + 2 * KB));
    static_assert((DEPTH - 1) * (2 * PB + 2 * KB) < 64, "vmcnt is a 6-bit counter");
    auto step = [&](int cb, auto J) __attribute__((always_inline)) {
        constexpr int j = decltype(J)::value;
        load_w(min(cb + DEPTH - 1, CiB - 1), wr[(j + DEPTH - 1) % DEPTH]);
        load_x(min(cb + DEPTH - 1, CiB - 1), xr[(j + DEPTH - 1) % DEPTH]);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(kWaitOlder);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < 8; ++q)
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) {
                    const float a = q < 4 ? wr[j][kb][0][q] : wr[j][kb][1][q - 4];
                    const float b = q < 4 ? xr[j][pb][0][q] : xr[j][pb][1][q - 4];
                    acc[kb][pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[kb][pb], 0, 0, 0);
                }
        __builtin_amdgcn_sched_barrier(0);
    };
    // whole rotations of the register slots without any branch inside, then the remaining steps
    int cb0 = 0;
    for (; cb0 + DEPTH <= CiB; cb0 += DEPTH)
        static_for<0, DEPTH>([&](auto J) __attribute__((always_inline)) { step(cb0 + decltype(J)::value, J); });
    static_for<0, DEPTH - 1>([&](auto J) __attribute__((always_inline)) {
        if (cb0 + decltype(J)::value < CiB) step(cb0 + decltype(J)::value, J);
    });

    // D layout of a 32x32 block: column (pixel) = lane % 32, row (channel) = 8*(r/4) + 4*(lane/32) + r%4:
    // four consecutive channels per group of 4 accumulators, one 16-byte store each
    const int Ko = KoB * kBlk;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int k = (kg * KB + kb) * 32 + 8 * gq + 4 * half;
                if (pvalid[pb] && k < Ko) {
                    const float4 v = make_float4(acc[kb][pb][4 * gq], acc[kb][pb][4 * gq + 1],
                                                 acc[kb][pb][4 * gq + 2], acc[kb][pb][4 * gq + 3]);
                    *reinterpret_cast<float4 *>(out + obase[pb] + (size_t)(k / kBlk) * plane + k % kBlk) = v;
                }
            }
}

template <int PB, int KB, int DEPTH>
hipError_t launch_pw(const Geom &g, const float *in, const float *wd, float *out, hipStream_t s)
{
    const int HW = g.Ho * g.Wo;
    const long long total_px = (long long)g.N * HW;
    const int kgroups = ceil_div(g.Ko, 32 * KB);
    const long long pgroups = (total_px + 4 * 32 * PB - 1) / (4 * 32 * PB);
    const long long blocks = (pgroups + 7) / 8 * 8 * kgroups;
    if (blocks > 0x7fffffffLL || total_px > 0x7fffff00LL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((pw_dense_kernel<PB, KB, DEPTH>), dim3((unsigned)blocks), dim3(256), 0, s, (int)total_px, HW,
                       g.Ci / kBlk, g.Ko / kBlk, in, wd, out, kgroups, g.sel, g.thr);
    return hipGetLastError();
}

// Variant for layers whose filters fit in LDS (at most 16 K elements: 256 -> 64, 64 -> 256, 64 -> 64,
// 128 -> 128: the bandwidth-bound 1x1 layers of the 56x56 ResNet stage, 25 flop/B against a ridge of 20).
// Time is lost there in four ways, and the structure answers each:
//  * one persistent workgroup of 8 wavefronts per compute unit copies the whole filter matrix into LDS
//    once, straight from the library layout with 16-byte coalesced reads, while the input of its first
//    tiles is already in flight;
//  * a tile is 32 pixels (the columns of v_mfma_f32_32x32x2_f32); the output channels of a tile are split
//    over the SIMDs (KS parts of KBW 32-channel blocks each), so the unit of work of a SIMD is a KS-th of a
//    tile and 12.25 tiles per compute unit (N = 32, 56x56) cost 13/12.25 of the ideal instead of 16/12.25;
//    the wavefronts that share a tile read the same input lines (one fetch from memory, the rest L1 hits);
//  * the channel loop runs on across tiles: a step (tile, channel block) requests the input of the step
//    DEPTH-1 = 3 later, which at the end of a tile belongs to the wavefront's next tile, so the load
//    queue does not drain between tiles.
// The two wavefronts of a SIMD take alternate tiles, so one's stores overlap the other's MFMAs.
// Measured on the 56x56 layers at N = 32 (128.5 MB per launch, 3.29 GF): 36 us for 256 -> 64 and 42 us
// for 64 -> 256 (45 and 58 us for the form this replaces).  The same kernel without its MFMAs takes 24-26 us
// (5 TB/s, the rate of a device-to-device copy), without its stores 34.5 us: the matrix pipe at its
// sustained rate is the longer of the two legs, and the stores of the layers that write four times what
// they read cost another 8 us on top.  The cause of those 8 us is not the order in which a wavefront's
// loads and stores complete (one counter tracks both, so a wait for loaded data can end up waiting for
// stores issued before it): a schedule in which the steps of a tile never wait behind stores (all of
// the next tile's input requested during the current tile, one wait for everything right before the
// stores) was measured and takes the same time.
// Measured and dropped: 7 and 15 blocks in flight (1-6 us slower: a wavefront has only 13 to 50 steps of
// work), four wavefronts per SIMD (4-8 us slower), filters of the next step read from LDS ahead of the
// MFMAs (4 us slower on 64 -> 256), streaming (non-temporal) stores (12 us slower).
// The steps are fully unrolled over a rotation of the DEPTH register slots and the first tile is peeled,
// so the wait the compiler places before each use counts exactly the loads issued since the request.
template <int KB, int KS, int CIB>
__global__ __launch_bounds__(512, 2) void pw_dense_lds_kernel(int total_px, int HW, const float *__restrict__ in,
                                                              const float *__restrict__ w, int transpose,
                                                              float *__restrict__ out, int tiles_per_wg,
                                                              const unsigned *sel, unsigned thr)
{
    constexpr int DEPTH = 4, WPS = 2;               // channel blocks in flight; wavefronts per SIMD
    constexpr int KBW = KB / KS, PS = 4 / KS;       // blocks per wavefront; tiles the four SIMDs work on at a time
    constexpr int KoB = KB * 2, Ko = KB * 32;
    constexpr int TPB = CIB >= DEPTH ? 1 : DEPTH / CIB;         // tiles per unrolled body (a whole number of rotations)
    constexpr int AHEAD = (DEPTH - 1 + CIB - 1) / CIB;          // tiles the requests reach past the body
    constexpr int NP = TPB + AHEAD;
    static_assert((TPB * CIB) % DEPTH == 0, "a body is a whole number of slot rotations");
    if (form_deselected(sel, 1, thr)) return;
    extern __shared__ __attribute__((aligned(16))) float wl[];      // [cb][kb][q][lane][4 c]
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;
    const int l32 = lane % 32, half = lane / 32;
    const int simd = wave % 4, turn = wave / 4;     // wavefronts w, w + 4, ... share a SIMD
    const int kpart = simd % KS, phase = simd / KS;

    const size_t plane = (size_t)HW * kBlk;
    const int ntiles = (total_px + 31) / 32;
    const int t0 = blockIdx.x * tiles_per_wg, t1 = min(t0 + tiles_per_wg, ntiles);
    const int stride = WPS * PS;
    const int first = t0 + phase + PS * turn;
    const int cnt = first < t1 ? (t1 - first + stride - 1) / stride : 0;     // tiles of this wavefront

    // this lane's pixel of the wavefront's tile number k: lanes past the end of the image data take the last
    // pixel (they compute and store its values a second time), tile numbers past the last take the last tile
    // (its lines are requested once more and never used)
    auto pixel_of = [&](int k, int &n, int &p) __attribute__((always_inline)) {
        int gp = (first + min(k, cnt - 1) * stride) * 32 + l32;
        if (gp >= total_px) gp = total_px - 1;
        n = gp / HW;
        p = gp % HW;
    };
    auto input_of = [&](int k) __attribute__((always_inline)) {
        int n, p;
        pixel_of(k, n, p);
        return in + ((size_t)n * CIB * HW + p) * kBlk + half * 8;
    };
    const float *xin[NP];
    float4 xr[DEPTH][2];
    auto request = [&](auto TGT) __attribute__((always_inline)) {         // step TGT of the body -> its slot
        constexpr int tgt = decltype(TGT)::value;
        const float4 *px = reinterpret_cast<const float4 *>(xin[tgt / CIB] + (size_t)(tgt % CIB) * plane);
        xr[tgt % DEPTH][0] = px[0];
        xr[tgt % DEPTH][1] = px[1];
    };
    if (cnt > 0) {
#pragma unroll
        for (int i = 0; i < NP; ++i) xin[i] = input_of(i);
        static_for<0, DEPTH - 1>([&](auto J) __attribute__((always_inline)) { request(J); });
    }

    // Filter copy from the library layout [K/16][C/16][16 c][16 k]: LDS float4 (cb, kb, q, lane = (half, k % 32))
    // holds channels c = 16*cb + 8*half + 4*q + 0..3 of output channel k = 32*kb + lane % 32.  A thread reads
    // 16 bytes (4 consecutive k of one c); transpose = the BWI form, where the roles of the two channel
    // dimensions are exchanged and those 4 values are 4 consecutive c of one k.
    // All reads are requested before the first LDS write (one round trip to memory instead of one per 512 float4).
    {
        const float4 *src = reinterpret_cast<const float4 *>(w);
        constexpr int total4 = Ko * CIB * 4;
        constexpr int NT = 256 * WPS;
        constexpr int kFill = (total4 + NT - 1) / NT;
        float4 fv[kFill];
#pragma unroll
        for (int it = 0; it < kFill; ++it) {
            const int i = threadIdx.x + it * NT;
            fv[it] = i < total4 ? src[i] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int it = 0; it < kFill; ++it) {
            const int i = threadIdx.x + it * NT;
            if (i >= total4) continue;
            const float4 v = fv[it];
            const int a = (i & 3) * 4, bq = (i >> 2) & 15;       // 4 values along the inner, one along the outer index
            if (!transpose) {
                const int cb = (i >> 6) % CIB, k0 = (i >> 6) / CIB * kBlk + a, ci = bq;
                float *d = wl + ((((cb * KB + k0 / 32) * 2 + (ci % 8) / 4) * 64 + (ci / 8) * 32 + k0 % 32) * 4 + ci % 4);
                d[0] = v.x; d[4] = v.y; d[8] = v.z; d[12] = v.w;
            } else {
                // the layer's [k_l block][c_l block]: Ko = its C, Ci = its K
                const int kb16 = (i >> 6) % KoB, cb = (i >> 6) / KoB, k = kb16 * kBlk + bq, ci = a;
                reinterpret_cast<float4 *>(wl)[((cb * KB + k / 32) * 2 + (ci % 8) / 4) * 64 + (ci / 8) * 32 + k % 32] = v;
            }
        }
    }
    __syncthreads();
    if (cnt == 0) return;
    const float4 *wl4 = reinterpret_cast<const float4 *>(wl) + lane + (size_t)kpart * KBW * 2 * 64;

    // filters of channel block cb for this wavefront's output channels
    auto filters = [&](int cb, float4 (&wv)[KBW][2]) __attribute__((always_inline)) {
#pragma unroll
        for (int kb = 0; kb < KBW; ++kb) {
            wv[kb][0] = wl4[((cb * KB + kb) * 2 + 0) * 64];
            wv[kb][1] = wl4[((cb * KB + kb) * 2 + 1) * 64];
        }
    };

    // TPB tiles starting at the wavefront's tile number k0 (the first exists)
    auto body = [&](int k0) __attribute__((always_inline)) {
        static_for<0, TPB>([&](auto TI) __attribute__((always_inline)) {
            constexpr int ti = decltype(TI)::value;
            if (ti > 0 && k0 + ti >= cnt) return;                       // uniform
            floatx16 acc[KBW];
#pragma unroll
            for (int kb = 0; kb < KBW; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[kb][r] = 0.f;
            static_for<0, CIB>([&](auto CB) __attribute__((always_inline)) {
                constexpr int cb = decltype(CB)::value, step = ti * CIB + cb;
                request(std::integral_constant<int, step + DEPTH - 1>{});
                float4 wv[KBW][2];
                filters(cb, wv);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = 0; q < 8; ++q)
#pragma unroll
                    for (int kb = 0; kb < KBW; ++kb) {
                        const float a = q < 4 ? wv[kb][0][q] : wv[kb][1][q - 4];
                        const float b = q < 4 ? xr[step % DEPTH][0][q] : xr[step % DEPTH][1][q - 4];
                        acc[kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[kb], 0, 0, 0);
                    }
                __builtin_amdgcn_sched_barrier(0);
            });
            // D layout of a 32x32 block: column (pixel) = lane % 32, row (channel) = 8*(r/4) + 4*(lane/32) + r%4
            int n, p;
            pixel_of(k0 + ti, n, p);
            float *yout = out + ((size_t)n * KoB * HW + p) * kBlk;
#pragma unroll
            for (int kb = 0; kb < KBW; ++kb)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int k = (kpart * KBW + kb) * 32 + 8 * gq + 4 * half;
                    const float4 v = make_float4(acc[kb][4 * gq], acc[kb][4 * gq + 1], acc[kb][4 * gq + 2], acc[kb][4 * gq + 3]);
                    *reinterpret_cast<float4 *>(yout + (size_t)(k / kBlk) * plane + k % kBlk) = v;
                }
            __builtin_amdgcn_sched_barrier(0);
        });
        // the tiles the next body works on and requests from
#pragma unroll
        for (int i = 0; i < NP; ++i) xin[i] = i + TPB < NP ? xin[i + TPB] : input_of(k0 + TPB + i);
    };

    body(0);                                            // after the prologue: no stores among the requests in flight
    for (int k0 = TPB; k0 < cnt; k0 += TPB) body(k0);
}

constexpr size_t kPwLdsBytes = 96 * 1024;       // more than half the LDS of a compute unit: one workgroup each

template <int KB, int KS, int CIB>
hipError_t launch_pw_lds(const Geom &g, bool transpose, const float *in, const float *w, float *out, hipStream_t s)
{
    const int HW = g.Ho * g.Wo;
    const long long total_px = (long long)g.N * HW;
    const long long ntiles = (total_px + 31) / 32;
    // one workgroup per compute unit, each with a contiguous share of the tiles
    const int tiles_per_wg = (int)((ntiles + 255) / 256);
    const long long blocks = (ntiles + tiles_per_wg - 1) / tiles_per_wg;
    auto kern = pw_dense_lds_kernel<KB, KS, CIB>;
    // More than 48 KB of dynamic LDS has to be allowed once per kernel and device; done on the first
    // call on that device, outside any launch sequence a caller may be capturing into a graph later.
    {
        static bool allowed[kMaxDevices] = {};
        int devid = 0;
        hipError_t e = hipGetDevice(&devid);
        if (e != hipSuccess) return e;
        if (devid < 0 || devid >= kMaxDevices) return hipErrorInvalidDevice;
        if (!allowed[devid]) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)kPwLdsBytes);
            if (e != hipSuccess) return e;
            allowed[devid] = true;
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(512), kPwLdsBytes, s, (int)total_px, HW, in, w,
                       transpose ? 1 : 0, out, tiles_per_wg, g.sel, g.thr);
    return hipGetLastError();
}

}  // namespace

// 1x1 layers whose filters fit in 64 KB of LDS, with 64, 128 or 256 output channels, and that have enough
// pixels to occupy the chip: computed straight from the library filter layout.
bool pw_dense_direct_supported(const Geom &g)
{
    if (g.R != 1 || g.S != 1 || g.sw != 1 || g.sh != 1 || g.uw != 1 || g.uh != 1 || g.pw != 0 || g.ph != 0) return false;
    const long long total_px = (long long)g.N * g.Ho * g.Wo;
    const bool shape = (g.Ko == 64 && (g.Ci == 64 || g.Ci == 128 || g.Ci == 256)) ||
                       (g.Ko == 128 && (g.Ci == 64 || g.Ci == 128)) || (g.Ko == 256 && g.Ci == 64);
    return shape && total_px >= 8192 && total_px <= 0x7fffff00LL;
}

hipError_t launch_pw_dense_direct(const Geom &g, bool transpose, const float *in, const float *w, float *out,
                                  hipStream_t s)
{
    if (g.Ko == 64) {
        if (g.Ci == 64) return launch_pw_lds<2, 2, 4>(g, transpose, in, w, out, s);
        if (g.Ci == 128) return launch_pw_lds<2, 2, 8>(g, transpose, in, w, out, s);
        return launch_pw_lds<2, 2, 16>(g, transpose, in, w, out, s);
    }
    if (g.Ko == 128) {
        if (g.Ci == 64) return launch_pw_lds<4, 4, 4>(g, transpose, in, w, out, s);
        return launch_pw_lds<4, 4, 8>(g, transpose, in, w, out, s);
    }
    return launch_pw_lds<8, 4, 4>(g, transpose, in, w, out, s);
}

// Requires fwd_dense_supported(g) with R = S = 1 (unit stride, no padding: Ho = Hi, Wo = Wi) and the
// filter copy of launch_reformat_filters, whose output channels are padded to a multiple of 128.
hipError_t launch_pw_dense(const Geom &g, const float *in, const float *wd, float *out, hipStream_t s)
{
    const long long total_px = (long long)g.N * g.Ho * g.Wo;
    // Tile choice (measured on the 1x1 shapes of Table 1 at N = 32): the largest tile that still
    // yields about one wavefront per SIMD (1024 on the chip); layers with at most 64 output channels
    // are bandwidth-bound and do best with the most wavefronts in flight.
    const int cand[6][2] = {{2, 4}, {1, 4}, {2, 2}, {1, 2}, {2, 1}, {1, 1}};
    int pb = 1, kb = 1;
    if (g.Ko > 64)
        for (const auto &c : cand) {
            if (32 * c[1] > ceil_div(g.Ko, 32) * 32) continue;
            const long long waves = (total_px + 32 * c[0] - 1) / (32 * c[0]) * ceil_div(g.Ko, 32 * c[1]);
            if (waves >= 768) { pb = c[0]; kb = c[1]; break; }
        }
    if (kb == 1) return pb == 1 ? launch_pw<1, 1, 4>(g, in, wd, out, s) : launch_pw<2, 1, 4>(g, in, wd, out, s);
    if (kb == 2) return pb == 1 ? launch_pw<1, 2, 4>(g, in, wd, out, s) : launch_pw<2, 2, 4>(g, in, wd, out, s);
    return pb == 1 ? launch_pw<1, 4, 3>(g, in, wd, out, s) : launch_pw<2, 4, 3>(g, in, wd, out, s);
}

}  // namespace st
