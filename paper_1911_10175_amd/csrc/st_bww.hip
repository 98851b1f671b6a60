// Filter-gradient kernels (BWW), unit stride: zero-skipping (vector ALUs) and dense (matrix cores).
//
// Mapping of SparseTrain Sec. 3.4 (Alg. 4-5) onto a CDNA wavefront:
//  * The filter-gradient accumulators are stationary (Sec. 3.4: T gradient vectors stay in
//    registers for the whole sweep): a wavefront owns 64 output channels (one per lane) times
//    16 input channels times R*S taps = 144 registers per lane for a 3x3 filter.
//  * The tested operand is the input x.  One pixel's 16-channel block is 64 contiguous bytes in
//    the blocked layout, fetched with one scalar load, so each channel value sits in a scalar
//    register: the zero test is a scalar compare, the skip a scalar branch over R*S multiply-
//    adds, and the non-zero value is the scalar operand of those multiply-adds (the broadcast
//    of Alg. 5).  The paper vectorises this test along the minibatch because its vector
//    register holds 16 values of one operand; a wavefront has separate scalar registers, so the
//    test runs along the channel block and the layout needs no minibatch transposition.
//  * The other operand, dy at the R*S neighbouring output pixels, is a vector over the lane's
//    output channel read from an LDS tile that the 4 wavefronts of a workgroup (4 different
//    16-channel input blocks) share.
//  * The sum over the minibatch and the image is split over workgroups; each writes a partial
//    gradient to the workspace and a second kernel adds the partials in a fixed order
//    (Sec. 3.4, accumulation of partial results at the end of a sweep), so results are
//    deterministic without floating-point atomics.
#include "st_common.hpp"

namespace st {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ size_t act_off(int n, int cb, int h, int w, int CB, int H, int W)
{
    return ((((size_t)n * CB + cb) * H + h) * W + w) * kBlk;
}

// x != 0 for a wavefront-uniform value, decided on the scalar unit: clearing the sign bit leaves
// zero exactly for +0 and -0 (denormals and NaNs count as non-zero).  The asm keeps the compiler
// from turning the integer test back into a vector float compare.
__device__ __forceinline__ bool scalar_nonzero(float v)
{
    unsigned mag;
    asm volatile("s_and_b32 %0, %1, 0x7fffffff" : "=s"(mag) : "s"(__float_as_uint(v)) : "scc");
    return mag != 0u;
}

// 16 channels of input pixel q of the tile (clamped into the image), wavefront-uniform address
__device__ __forceinline__ void load_x16(const float *__restrict__ x, int n, int cb, int ih0, int iw0,
                                         int q, int TW, int CB, int H, int W, float (&dst)[kBlk])
{
    const int ih = min(ih0 + q / TW, H - 1), iw = min(iw0 + q % TW, W - 1);
    const float4 *p = reinterpret_cast<const float4 *>(x + act_off(n, cb, ih, iw, CB, H, W));
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float4 v = p[j];
        dst[4 * j + 0] = v.x; dst[4 * j + 1] = v.y; dst[4 * j + 2] = v.z; dst[4 * j + 3] = v.w;
    }
}

// dy at the R*S output pixels that read input pixel q of the tile, for this lane's channel
template <int R, int S, int HW>
__device__ __forceinline__ void load_dy_taps(const float *dyT, int q, int TW, int lane, float (&dst)[S * R])
{
    const int a = q / TW, b = q % TW;
#pragma unroll
    for (int v = 0; v < S; ++v)
#pragma unroll
        for (int u = 0; u < R; ++u)
            dst[v * R + u] = dyT[((a + S - 1 - v) * HW + (b + R - 1 - u)) * 64 + lane];
}

struct BwwArgs {
    int N, C, K, H, W, OH, OW, pw, ph;
    int tiles_w, tiles_h;      // tiles over the input image (sparse) / the output image (dense)
    int units;                 // N * tiles_h * tiles_w
    int splits;                // partial sums; gridDim.x
    int cgroups;               // ceil(C/64)
};

template <int R, int S, int TH, int TW>
struct BwwCfg {
    static constexpr int HH = TH + S - 1, HW = TW + R - 1, HP = HH * HW;
};

// ------------------------------------------------------------------------------------------
// zero-skipping kernel: tiles run over the INPUT image; LDS holds the dy halo of the tile
// ------------------------------------------------------------------------------------------
template <int R, int S, int TH, int TW>
__global__ __launch_bounds__(256) void bww_sparse_kernel(BwwArgs A, const float *__restrict__ x,
                                                         const float *__restrict__ dy,
                                                         float *__restrict__ part)
{
    using Cfg = BwwCfg<R, S, TH, TW>;
    constexpr int HW = Cfg::HW, HP = Cfg::HP;
    __shared__ __attribute__((aligned(16))) float dyT[HP * 64];

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int lane = threadIdx.x % kWave;
    const int split = blockIdx.x;
    const int kt = blockIdx.y / A.cgroups, cg = blockIdx.y % A.cgroups;
    const int CB = A.C / kBlk, KB = A.K / kBlk;
    const int cb = cg * 4 + wave;
    const bool wave_active = cb < CB;
    const int k = kt * 64 + lane;

    float acc[kBlk][S * R];
#pragma unroll
    for (int ci = 0; ci < kBlk; ++ci)
#pragma unroll
        for (int t = 0; t < S * R; ++t) acc[ci][t] = 0.f;

    const int u0 = (int)((long long)A.units * split / A.splits);
    const int u1 = (int)((long long)A.units * (split + 1) / A.splits);

    for (int unit = u0; unit < u1; ++unit) {
        int t = unit;
        const int tw = t % A.tiles_w; t /= A.tiles_w;
        const int th = t % A.tiles_h;
        const int n = t / A.tiles_h;
        const int ih0 = th * TH, iw0 = tw * TW;
        const int ohs = ih0 + A.ph - (S - 1), ows = iw0 + A.pw - (R - 1);

        __syncthreads();
        // stage dy[n, kt*64 .. +63, halo] as [pixel][64 k]; 16 float4 per pixel
        for (int idx = threadIdx.x; idx < HP * 16; idx += 256) {
            const int pix = idx >> 4, q = idx & 15;
            const int oh = ohs + pix / HW, ow = ows + pix % HW;
            const int kb = kt * 4 + (q >> 2);
            float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
            if (oh >= 0 && oh < A.OH && ow >= 0 && ow < A.OW && kb < KB)
                val = *reinterpret_cast<const float4 *>(dy + act_off(n, kb, oh, ow, KB, A.OH, A.OW) + (q & 3) * 4);
            *reinterpret_cast<float4 *>(dyT + pix * 64 + q * 4) = val;
        }
        __syncthreads();
        if (!wave_active) continue;

        // Software pipeline over the pixels of the tile: the scalar load of the next pixel's 16
        // channels and the LDS reads of its dy neighbourhood are issued before the multiply-adds
        // of the current pixel.  Coordinates are clamped for the loads (always in bounds); pixels
        // outside the image are skipped by the validity test.
        float xs[kBlk], dyv[S * R];
        load_x16(x, n, cb, ih0, iw0, 0, TW, CB, A.H, A.W, xs);
        load_dy_taps<R, S, HW>(dyT, 0, TW, lane, dyv);
        __builtin_amdgcn_s_waitcnt(0xC07F);
        for (int q = 0; q < TH * TW; ++q) {
            float xn[kBlk], dyn[S * R];
            const int qn = (q + 1 < TH * TW) ? q + 1 : q;
            load_x16(x, n, cb, ih0, iw0, qn, TW, CB, A.H, A.W, xn);
            load_dy_taps<R, S, HW>(dyT, qn, TW, lane, dyn);
            const bool valid = (ih0 + q / TW < A.H) && (iw0 + q % TW < A.W);
            if (valid) {
#pragma unroll
                for (int ci = 0; ci < kBlk; ++ci) {
                    if (scalar_nonzero(xs[ci])) {
#pragma unroll
                        for (int tp = 0; tp < S * R; ++tp) acc[ci][tp] = fmaf(xs[ci], dyv[tp], acc[ci][tp]);
                    }
                }
            }
            // the prefetched operands have had the whole pixel's arithmetic to arrive; waiting
            // here (lgkmcnt(0)) keeps the compiler from waiting for them before that arithmetic
            __builtin_amdgcn_s_waitcnt(0xC07F);
#pragma unroll
            for (int ci = 0; ci < kBlk; ++ci) xs[ci] = xn[ci];
#pragma unroll
            for (int tp = 0; tp < S * R; ++tp) dyv[tp] = dyn[tp];
        }
    }

    if (wave_active && k < A.K) {
        const int kb = k / kBlk, ki = k % kBlk;
        float *p = part + (size_t)split * A.K * A.C * (S * R) +
                   ((size_t)kb * CB + cb) * (S * R * kBlk * kBlk) + ki;
#pragma unroll
        for (int tp = 0; tp < S * R; ++tp)
#pragma unroll
            for (int ci = 0; ci < kBlk; ++ci) p[tp * (kBlk * kBlk) + ci * kBlk] = acc[ci][tp];
    }
}

// ------------------------------------------------------------------------------------------
// dense kernel: tiles run over the OUTPUT image; LDS holds the dy tile and the x halo.
// v_mfma_f32_32x32x2_f32 with rows = 32 input channels, columns = 32 output channels, reduction
// = 2 pixels per instruction; one accumulator block per filter tap.
// ------------------------------------------------------------------------------------------
template <int R, int S, int TH, int TW>
__global__ __launch_bounds__(256) void bww_dense_kernel(BwwArgs A, const float *__restrict__ x,
                                                        const float *__restrict__ dy,
                                                        float *__restrict__ part)
{
    using Cfg = BwwCfg<R, S, TH, TW>;
    constexpr int HW = Cfg::HW, HP = Cfg::HP, TP = TH * TW;
    static_assert(TW % 2 == 0, "pixel pairs must not straddle rows");
    __shared__ __attribute__((aligned(16))) float dyT[TP * 64];
    __shared__ __attribute__((aligned(16))) float xT[HP * 64];

    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
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

    for (int unit = u0; unit < u1; ++unit) {
        int t = unit;
        const int tw = t % A.tiles_w; t /= A.tiles_w;
        const int th = t % A.tiles_h;
        const int n = t / A.tiles_h;
        const int oh0 = th * TH, ow0 = tw * TW;
        const int ih0 = oh0 - A.ph, iw0 = ow0 - A.pw;

        __syncthreads();
        for (int idx = threadIdx.x; idx < TP * 16; idx += 256) {
            const int pix = idx >> 4, q = idx & 15;
            const int oh = oh0 + pix / TW, ow = ow0 + pix % TW;
            const int kb = kt * 4 + (q >> 2);
            float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
            if (oh < A.OH && ow < A.OW && kb < KB)
                val = *reinterpret_cast<const float4 *>(dy + act_off(n, kb, oh, ow, KB, A.OH, A.OW) + (q & 3) * 4);
            *reinterpret_cast<float4 *>(dyT + pix * 64 + q * 4) = val;
        }
        for (int idx = threadIdx.x; idx < HP * 16; idx += 256) {
            const int pix = idx >> 4, q = idx & 15;
            const int ih = ih0 + pix / HW, iw = iw0 + pix % HW;
            const int cb = cg * 4 + (q >> 2);
            float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
            if (ih >= 0 && ih < A.H && iw >= 0 && iw < A.W && cb < CB)
                val = *reinterpret_cast<const float4 *>(x + act_off(n, cb, ih, iw, CB, A.H, A.W) + (q & 3) * 4);
            *reinterpret_cast<float4 *>(xT + pix * 64 + q * 4) = val;
        }
        __syncthreads();

        for (int pp = 0; pp < TP / 2; ++pp) {
            const int p = 2 * pp + half;
            const int a = p / TW, b = p % TW;
            const float bv = dyT[p * 64 + kh * 32 + l32];                  // B[kk = half][j = k]
#pragma unroll
            for (int v = 0; v < S; ++v)
#pragma unroll
                for (int u = 0; u < R; ++u) {
                    const float av = xT[((a + v) * HW + (b + u)) * 64 + ch * 32 + l32];   // A[i = c][kk]
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

// dw[i] = sum over splits of part[s][i], in split order
__global__ __launch_bounds__(256) void bww_reduce_kernel(const float4 *__restrict__ part,
                                                         float4 *__restrict__ dw, size_t n4, int splits)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    float4 s = part[i];
    for (int p = 1; p < splits; ++p) {
        const float4 v = part[(size_t)p * n4 + i];
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    dw[i] = s;
}

constexpr int kSparseTH = 8, kSparseTW = 16;
constexpr int kDenseTH = 8, kDenseTW = 16;

BwwArgs make_args(const st_conv_desc &d, int TH, int TW, bool tiles_over_input)
{
    BwwArgs A;
    A.N = d.N; A.C = d.C; A.K = d.K; A.H = d.H; A.W = d.W;
    A.OH = d.H + 2 * d.pad_h - d.S + 1;
    A.OW = d.W + 2 * d.pad_w - d.R + 1;
    A.pw = d.pad_w; A.ph = d.pad_h;
    const int eh = tiles_over_input ? d.H : A.OH, ew = tiles_over_input ? d.W : A.OW;
    A.tiles_h = ceil_div(eh, TH);
    A.tiles_w = ceil_div(ew, TW);
    A.units = d.N * A.tiles_h * A.tiles_w;
    A.cgroups = ceil_div(d.C, 64);
    const int groups = ceil_div(d.K, 64) * A.cgroups;
    int splits = ceil_div(1024, groups);         // aim at >= 4 workgroups per compute unit
    if (splits > A.units) splits = A.units;
    if (splits < 1) splits = 1;
    A.splits = splits;
    return A;
}

size_t partial_bytes(const st_conv_desc &d, const BwwArgs &A)
{
    if (A.splits == 1) return 0;
    return (size_t)A.splits * d.K * d.C * d.S * d.R * sizeof(float);
}

hipError_t reduce(const st_conv_desc &d, const BwwArgs &A, const float *part, float *dw, hipStream_t s)
{
    if (A.splits == 1) return hipSuccess;
    const size_t n4 = (size_t)d.K * d.C * d.S * d.R / 4;
    hipLaunchKernelGGL(bww_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s,
                       reinterpret_cast<const float4 *>(part), reinterpret_cast<float4 *>(dw), n4, A.splits);
    return hipGetLastError();
}

}  // namespace

bool bww_fast_supported(const st_conv_desc &d)
{
    if (d.stride_w != 1 || d.stride_h != 1) return false;
    const long long units = (long long)d.N * ceil_div(d.H + 2 * d.pad_h, 8) * ceil_div(d.W + 2 * d.pad_w, 16);
    if (units > 0x7fffffffLL) return false;
    if (d.R == 3 && d.S == 3) return d.pad_w <= 2 && d.pad_h <= 2;
    if (d.R == 1 && d.S == 1) return d.pad_w == 0 && d.pad_h == 0;
    return false;
}

size_t bww_sparse_workspace(const st_conv_desc &d)
{
    return partial_bytes(d, make_args(d, kSparseTH, kSparseTW, true));
}

size_t bww_dense_workspace(const st_conv_desc &d)
{
    return partial_bytes(d, make_args(d, kDenseTH, kDenseTW, false));
}

hipError_t launch_bww_sparse(const st_conv_desc &d, const float *x, const float *dy, float *dw,
                             float *ws, hipStream_t s)
{
    const BwwArgs A = make_args(d, kSparseTH, kSparseTW, true);
    float *part = A.splits == 1 ? dw : ws;
    dim3 grid(A.splits, ceil_div(d.K, 64) * A.cgroups);
    if (d.R == 3)
        hipLaunchKernelGGL((bww_sparse_kernel<3, 3, kSparseTH, kSparseTW>), grid, dim3(256), 0, s, A, x, dy, part);
    else
        hipLaunchKernelGGL((bww_sparse_kernel<1, 1, kSparseTH, kSparseTW>), grid, dim3(256), 0, s, A, x, dy, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return reduce(d, A, part, dw, s);
}

hipError_t launch_bww_dense(const st_conv_desc &d, const float *x, const float *dy, float *dw,
                            float *ws, hipStream_t s)
{
    const BwwArgs A = make_args(d, kDenseTH, kDenseTW, false);
    float *part = A.splits == 1 ? dw : ws;
    dim3 grid(A.splits, ceil_div(d.K, 64) * A.cgroups);
    if (d.R == 3)
        hipLaunchKernelGGL((bww_dense_kernel<3, 3, kDenseTH, kDenseTW>), grid, dim3(256), 0, s, A, x, dy, part);
    else
        hipLaunchKernelGGL((bww_dense_kernel<1, 1, kDenseTH, kDenseTW>), grid, dim3(256), 0, s, A, x, dy, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return reduce(d, A, part, dw, s);
}

}  // namespace st
