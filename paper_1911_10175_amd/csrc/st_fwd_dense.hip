// Dense unit-stride correlation on the matrix cores: the control the zero-skipping kernels are
// measured against (the role the library's dense "direct" convolution plays in SparseTrain
// Sec. 4).  Used for FWD and, with transposed filters, for BWI.
//
// Implicit GEMM with v_mfma_f32_32x32x2_f32: rows = 32 output pixels, columns = 32 output
// channels, reduction = 2 input channels of one filter tap per instruction.  A wavefront owns an
// 8x8 pixel tile times 64 output channels (2x2 MFMA blocks, 64 accumulator registers).  The
// input halo of the tile for one 16-channel block is staged in a wavefront-private LDS region
// (zero padding is applied there once); for every tap the A operand is read from LDS at the
// shifted pixel, the B operand (filters) comes straight from global memory / L2 in the
// library's [K/16][C/16][S][R][16][16] layout.  No tests, no skipping.
#include "st_common.hpp"

namespace st {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ size_t act_off(int n, int cb, int h, int w, int CB, int H, int W)
{
    return ((((size_t)n * CB + cb) * H + h) * W + w) * kBlk;
}

template <int R, int S>
struct FwdDenseCfg {
    static constexpr int TH = 8, TW = 8;
    static constexpr int HH = TH + S - 1, HW = TW + R - 1, HP = HH * HW;
    static constexpr int XST = 20;          // floats per staged pixel (16 channels + 4 pad)
    static constexpr int WAVES = 4;
    static constexpr int KT = 64;
};

template <int R, int S>
__global__ __launch_bounds__(256, 4) void fwd_dense_kernel(Geom g, const float *__restrict__ in,
                                                        const float *__restrict__ f,
                                                        float *__restrict__ out,
                                                        int tiles_w, int tiles_h, int ktiles, int total)
{
    using Cfg = FwdDenseCfg<R, S>;
    constexpr int TH = Cfg::TH, TW = Cfg::TW, HW = Cfg::HW, HP = Cfg::HP, XST = Cfg::XST;
    __shared__ __attribute__((aligned(16))) float lds_all[Cfg::WAVES][HP * XST];

    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int wid = blockIdx.x * Cfg::WAVES + wave;
    if (wid >= total) return;                       // no block-level barrier is used below
    float *lds = lds_all[wave];

    int t = wid;
    const int kt = t % ktiles; t /= ktiles;
    const int tw = t % tiles_w; t /= tiles_w;
    const int th = t % tiles_h;
    const int n = t / tiles_h;
    const int oh0 = th * TH, ow0 = tw * TW;
    const int ih0 = oh0 - g.ph, iw0 = ow0 - g.pw;
    const int CiB = g.Ci / kBlk, KoB = g.Ko / kBlk;

    const int l32 = lane % 32, half = lane / 32;

    floatx16 acc[2][2];
#pragma unroll
    for (int pb = 0; pb < 2; ++pb)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[pb][kb][r] = 0.f;

    // B operand: lane supplies filter element (k = kt*64 + kb2*32 + l32, c = j + 8*half), j = 0..7
    const float *fp[2];
    bool kact[2];
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2) {
        const int k = kt * Cfg::KT + kb2 * 32 + l32;
        kact[kb2] = k < g.Ko;
        const int kb = kact[kb2] ? k / kBlk : 0;
        fp[kb2] = f + (size_t)kb * CiB * (S * R * kBlk * kBlk) + (half * 8) * kBlk + (k % kBlk);
    }
    // A operand: lane supplies input (pixel = pb*32 + l32 of the tile, channels half*8 .. half*8+7)
    int apix[2];
#pragma unroll
    for (int pb = 0; pb < 2; ++pb) {
        const int p = pb * 32 + l32;
        apix[pb] = (p / TW) * HW + (p % TW);
    }

    for (int cb = 0; cb < CiB; ++cb) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int jj = 0; jj < (HP * 4 + 63) / 64; ++jj) {
            const int idx = jj * kWave + lane;
            const int pix = idx >> 2, q = idx & 3;
            if (pix < HP) {
                const int a = pix / HW, b = pix % HW;
                const int ih = ih0 + a, iw = iw0 + b;
                float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
                if (ih >= 0 && ih < g.Hi && iw >= 0 && iw < g.Wi)
                    val = *reinterpret_cast<const float4 *>(in + act_off(n, cb, ih, iw, CiB, g.Hi, g.Wi) + q * 4);
                *reinterpret_cast<float4 *>(lds + pix * XST + q * 4) = val;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

#pragma unroll
        for (int v = 0; v < S; ++v)
#pragma unroll
            for (int u = 0; u < R; ++u) {
                const int tap = v * R + u;
                float a[2][8], b[2][8];
#pragma unroll
                for (int kb2 = 0; kb2 < 2; ++kb2) {
                    const float *p = fp[kb2] + ((size_t)cb * (S * R) + tap) * (kBlk * kBlk);
#pragma unroll
                    for (int j = 0; j < 8; ++j) b[kb2][j] = p[j * kBlk];
                }
#pragma unroll
                for (int pb = 0; pb < 2; ++pb) {
                    const float *p = lds + (apix[pb] + v * HW + u) * XST + half * 8;
                    const float4 lo = *reinterpret_cast<const float4 *>(p);
                    const float4 hi = *reinterpret_cast<const float4 *>(p + 4);
                    a[pb][0] = lo.x; a[pb][1] = lo.y; a[pb][2] = lo.z; a[pb][3] = lo.w;
                    a[pb][4] = hi.x; a[pb][5] = hi.y; a[pb][6] = hi.z; a[pb][7] = hi.w;
                }
#pragma unroll
                for (int j = 0; j < 8; ++j)
#pragma unroll
                    for (int pb = 0; pb < 2; ++pb)
#pragma unroll
                        for (int kb2 = 0; kb2 < 2; ++kb2)
                            acc[pb][kb2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[pb][j], b[kb2][j],
                                                                               acc[pb][kb2], 0, 0, 0);
            }
    }

    // D layout of the 32x32 block: column = lane % 32, row = 8*(r/4) + 4*(lane/32) + r%4
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2) {
        if (!kact[kb2]) continue;
        const int k = kt * Cfg::KT + kb2 * 32 + l32;
        const int kb = k / kBlk, ki = k % kBlk;
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int p = pb * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                const int oh = oh0 + p / TW, ow = ow0 + p % TW;
                if (oh < g.Ho && ow < g.Wo)
                    out[act_off(n, kb, oh, ow, KoB, g.Ho, g.Wo) + ki] = acc[pb][kb2][r];
            }
    }
}

template <int R, int S>
hipError_t launch_cfg(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    using Cfg = FwdDenseCfg<R, S>;
    const int tiles_w = ceil_div(g.Wo, Cfg::TW), tiles_h = ceil_div(g.Ho, Cfg::TH);
    const int ktiles = ceil_div(g.Ko, Cfg::KT);
    const long long total = (long long)tiles_w * tiles_h * ktiles * g.N;
    if (total > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)((total + Cfg::WAVES - 1) / Cfg::WAVES));
    hipLaunchKernelGGL((fwd_dense_kernel<R, S>), grid, dim3(256), 0, s, g, in, f, out, tiles_w, tiles_h,
                       ktiles, (int)total);
    return hipGetLastError();
}

}  // namespace

bool fwd_dense_supported(const Geom &g)
{
    if (g.sw != 1 || g.sh != 1) return false;
    if (g.R == 3 && g.S == 3) return g.pw <= 2 && g.ph <= 2;
    if (g.R == 1 && g.S == 1) return g.pw == 0 && g.ph == 0;
    return false;
}

hipError_t launch_fwd_dense(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    if (g.R == 3 && g.S == 3) return launch_cfg<3, 3>(g, in, f, out, s);
    if (g.R == 1 && g.S == 1) return launch_cfg<1, 1>(g, in, f, out, s);
    return hipErrorInvalidValue;
}

}  // namespace st
