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

// Variant for layers whose filters fit in LDS (at most 16 K elements, e.g. 256 -> 64, 64 -> 256,
// 64 -> 64: the bandwidth-bound 1x1 layers of the 56x56 ResNet stage).  A workgroup copies the whole
// filter matrix into LDS once and then walks pixel tiles of 32 pixels per wavefront; a wavefront
// computes all K output channels of its tile, so an input element is fetched from memory exactly
// once and the only vector-memory traffic in the loop is the input itself; the filter operand is
// read from LDS with 16-byte reads that touch consecutive addresses in consecutive lanes.
template <int KB, int DEPTH>
__global__ __launch_bounds__(256, 2) void pw_dense_lds_kernel(int total_px, int HW, int CiB, int KoB,
                                                              const float *__restrict__ in,
                                                              const float *__restrict__ w, int transpose,
                                                              float *__restrict__ out, const unsigned *sel,
                                                              unsigned thr)
{
    if (form_deselected(sel, 1, thr)) return;
    extern __shared__ __attribute__((aligned(16))) float wl[];      // [cb][kb][q][lane][4 c]
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;
    const int l32 = lane % 32, half = lane / 32;

    // Filter copy straight from the library layout [K/16][C/16][16 c][16 k] (no reformatting pass):
    // LDS float4 (cb, kb, q, lane = (half, k % 32)) holds channels c = 16*cb + 8*half + 4*q + 0..3 of
    // output channel k = 32*kb + lane % 32; transpose = the BWI form, where the roles of the two
    // channel dimensions are exchanged.  Output channels beyond Ko are zero.
    {
        float4 *dst = reinterpret_cast<float4 *>(wl);
        const int total4 = KB * CiB * 128;
        const int Ko = KoB * kBlk;
        for (int i = threadIdx.x; i < total4; i += 256) {
            const int sl32 = i & 31, shalf = (i >> 5) & 1, q = (i >> 6) & 1;
            const int blk = i >> 7, kb = blk % KB, cb = blk / KB;
            const int k = kb * 32 + sl32, c0 = cb * kBlk + shalf * 8 + q * 4;
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            if (k < Ko) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int c = c0 + e;
                    v[e] = transpose ? w[((size_t)(c / kBlk) * KoB + k / kBlk) * (kBlk * kBlk) + (k % kBlk) * kBlk + c % kBlk]
                                     : w[((size_t)(k / kBlk) * CiB + c / kBlk) * (kBlk * kBlk) + (c % kBlk) * kBlk + k % kBlk];
                }
            }
            dst[i] = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
    __syncthreads();
    const float4 *wl4 = reinterpret_cast<const float4 *>(wl) + lane;

    const size_t plane = (size_t)HW * kBlk;
    const int ntiles = (total_px + 31) / 32;
    const int Ko = KoB * kBlk;
    constexpr int kWaitOlder = vmcnt_imm((DEPTH - 1) * 2);

    for (int tile = blockIdx.x * 4 + wave; tile < ntiles; tile += gridDim.x * 4) {
        int gp = tile * 32 + l32;
        const bool pvalid = gp < total_px;
        if (!pvalid) gp = total_px - 1;
        const int n = gp / HW, p = gp % HW;
        const float *xin = in + ((size_t)n * CiB * HW + p) * kBlk + half * 8;
        float *yout = out + ((size_t)n * KoB * HW + p) * kBlk;

        floatx16 acc[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[kb][r] = 0.f;

        float4 xr[DEPTH][2];
        static_for<0, DEPTH - 1>([&](auto J) __attribute__((always_inline)) {
            constexpr int j = decltype(J)::value;
            const float4 *px = reinterpret_cast<const float4 *>(xin + (size_t)min(j, CiB - 1) * plane);
            xr[j][0] = px[0];
            xr[j][1] = px[1];
        });
        // CiB is a multiple of DEPTH (checked by the host): whole rotations of the register slots
        for (int cb0 = 0; cb0 < CiB; cb0 += DEPTH)
            static_for<0, DEPTH>([&](auto J) __attribute__((always_inline)) {
                constexpr int j = decltype(J)::value;
                const int cb = cb0 + j;
                const float4 *px = reinterpret_cast<const float4 *>(xin + (size_t)min(cb + DEPTH - 1, CiB - 1) * plane);
                xr[(j + DEPTH - 1) % DEPTH][0] = px[0];
                xr[(j + DEPTH - 1) % DEPTH][1] = px[1];
                float4 wv[KB][2];
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) {
                    wv[kb][0] = wl4[((cb * KB + kb) * 2 + 0) * 64];
                    wv[kb][1] = wl4[((cb * KB + kb) * 2 + 1) * 64];
                }
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_s_waitcnt(kWaitOlder);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = 0; q < 8; ++q)
#pragma unroll
                    for (int kb = 0; kb < KB; ++kb) {
                        const float a = q < 4 ? wv[kb][0][q] : wv[kb][1][q - 4];
                        const float b = q < 4 ? xr[j][0][q] : xr[j][1][q - 4];
                        acc[kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[kb], 0, 0, 0);
                    }
                __builtin_amdgcn_sched_barrier(0);
            });

#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int k = kb * 32 + 8 * gq + 4 * half;
                if (pvalid && k < Ko) {
                    const float4 v = make_float4(acc[kb][4 * gq], acc[kb][4 * gq + 1], acc[kb][4 * gq + 2],
                                                 acc[kb][4 * gq + 3]);
                    *reinterpret_cast<float4 *>(yout + (size_t)(k / kBlk) * plane + k % kBlk) = v;
                }
            }
    }
}

template <int KB>
hipError_t launch_pw_lds(const Geom &g, bool transpose, const float *in, const float *w, float *out, hipStream_t s)
{
    const int HW = g.Ho * g.Wo;
    const long long total_px = (long long)g.N * HW;
    const int CiB = g.Ci / kBlk;
    const size_t lds = (size_t)KB * 32 * g.Ci * sizeof(float);
    const long long ntiles = (total_px + 31) / 32;
    // two workgroups per compute unit (LDS permitting); fewer when there are not enough tiles
    long long blocks = 512;
    if (blocks * 4 > ntiles) blocks = (ntiles + 3) / 4;
    auto kern = pw_dense_lds_kernel<KB, 4>;
    // More than 48 KB of dynamic LDS has to be allowed once per kernel and device; done on the first
    // call on that device (with 64 KB, the most a supported filter matrix takes), outside any launch
    // sequence a caller may be capturing into a graph later.
    if (lds > 48 * 1024) {
        static bool allowed[kMaxDevices] = {};
        int devid = 0;
        hipError_t e = hipGetDevice(&devid);
        if (e != hipSuccess) return e;
        if (devid < 0 || devid >= kMaxDevices) return hipErrorInvalidDevice;
        if (!allowed[devid]) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
            if (e != hipSuccess) return e;
            allowed[devid] = true;
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), lds, s, (int)total_px, HW, CiB, g.Ko / kBlk, in, w,
                       transpose ? 1 : 0, out, g.sel, g.thr);
    return hipGetLastError();
}

}  // namespace

// 1x1 layers whose filters fit in LDS (64 KB with the output channels padded to 64, 128 or 256) and
// that have enough pixels to occupy the chip: computed straight from the library filter layout.
bool pw_dense_direct_supported(const Geom &g)
{
    if (g.R != 1 || g.S != 1 || g.sw != 1 || g.sh != 1 || g.uw != 1 || g.uh != 1 || g.pw != 0 || g.ph != 0) return false;
    const int kb_all = g.Ko <= 64 ? 2 : (g.Ko <= 128 ? 4 : 8);
    const long long total_px = (long long)g.N * g.Ho * g.Wo;
    return g.Ko <= 256 && (size_t)kb_all * 32 * g.Ci * sizeof(float) <= 64 * 1024 && (g.Ci / kBlk) % 4 == 0 &&
           total_px >= 8192 && total_px <= 0x7fffff00LL;
}

hipError_t launch_pw_dense_direct(const Geom &g, bool transpose, const float *in, const float *w, float *out,
                                  hipStream_t s)
{
    if (g.Ko <= 64) return launch_pw_lds<2>(g, transpose, in, w, out, s);
    if (g.Ko <= 128) return launch_pw_lds<4>(g, transpose, in, w, out, s);
    return launch_pw_lds<8>(g, transpose, in, w, out, s);
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
