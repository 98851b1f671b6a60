// Generic kernels: every geometry the API accepts (any stride, padding, filter size).
//
// They are the fall-back for shapes the tiled unit-stride kernels do not cover.  One wavefront
// owns one output location and up to 64 channels of the vectorised dimension (one channel per
// lane), so the tested operand is a single value shared by the whole wavefront: the zero test
// is a scalar compare and a taken branch skips the multiply-add for all lanes at once.  This is
// the direct analogue of the paper's broadcast-scalar times channel-vector FMA with the zero
// test in front of it (SparseTrain Sec. 3.1, Alg. 1; Sec. 3.4, Alg. 4), written per output
// (gather form) so that no two wavefronts update the same element.
#include "st_common.hpp"
#include "st_filter_copies.hpp"

namespace st {
namespace {

__device__ __forceinline__ size_t flt_off(int kb, int cb, int v, int u, int CB, int S, int R)
{
    return ((((size_t)kb * CB + cb) * S + v) * R + u) * (kBlk * kBlk);
}

// y[n,k,oh,ow] for k = 64*blockIdx.y + lane
template <bool SPARSE>
__global__ __launch_bounds__(64) void generic_fwd_kernel(st_conv_desc d, int OH, int OW,
                                                         const float *__restrict__ x,
                                                         const float *__restrict__ w,
                                                         float *__restrict__ y, const unsigned *sel, unsigned thr)
{
    if (form_deselected(sel, SPARSE ? 0 : 1, thr)) return;
    const int lane = threadIdx.x;
    const int k = blockIdx.y * kWave + lane;
    const int ow = blockIdx.x % OW, oh = blockIdx.x / OW, n = blockIdx.z;
    const int CB = d.C / kBlk;
    const bool active = k < d.K;
    const int kb = active ? k / kBlk : 0, ki = k % kBlk;
    float acc = 0.f;
    for (int v = 0; v < d.S; ++v) {
        const int ih = oh * d.stride_h - d.pad_h + v;
        if (ih < 0 || ih >= d.H) continue;
        for (int u = 0; u < d.R; ++u) {
            const int iw = ow * d.stride_w - d.pad_w + u;
            if (iw < 0 || iw >= d.W) continue;
            for (int cb = 0; cb < CB; ++cb) {
                const float *xp = x + act_off(n, cb, ih, iw, CB, d.H, d.W);
                const float *wp = w + flt_off(kb, cb, v, u, CB, d.S, d.R) + ki;
                for (int ci = 0; ci < kBlk; ++ci) {
                    const float xv = xp[ci];            // same address in every lane
                    if (SPARSE && !(xv != 0.f)) continue;
                    acc = fmaf(xv, wp[ci * kBlk], acc);
                }
            }
        }
    }
    if (active) y[act_off(n, kb, oh, ow, d.K / kBlk, OH, OW) + ki] = acc;
}

// dx[n,c,ih,iw] for c = 64*blockIdx.y + lane
template <bool SPARSE>
__global__ __launch_bounds__(64) void generic_bwi_kernel(st_conv_desc d, int OH, int OW,
                                                         const float *__restrict__ dy,
                                                         const float *__restrict__ w,
                                                         float *__restrict__ dx, const unsigned *sel, unsigned thr)
{
    if (form_deselected(sel, SPARSE ? 0 : 1, thr)) return;
    const int lane = threadIdx.x;
    const int c = blockIdx.y * kWave + lane;
    const int iw = blockIdx.x % d.W, ih = blockIdx.x / d.W, n = blockIdx.z;
    const int CB = d.C / kBlk, KB = d.K / kBlk;
    const bool active = c < d.C;
    const int cb = active ? c / kBlk : 0, ci = c % kBlk;
    float acc = 0.f;
    for (int v = 0; v < d.S; ++v) {
        const int th = ih + d.pad_h - v;
        if (th < 0 || th % d.stride_h) continue;
        const int oh = th / d.stride_h;
        if (oh >= OH) continue;
        for (int u = 0; u < d.R; ++u) {
            const int tw = iw + d.pad_w - u;
            if (tw < 0 || tw % d.stride_w) continue;
            const int ow = tw / d.stride_w;
            if (ow >= OW) continue;
            for (int kb = 0; kb < KB; ++kb) {
                const float *gp = dy + act_off(n, kb, oh, ow, KB, OH, OW);
                const float *wp = w + flt_off(kb, cb, v, u, CB, d.S, d.R) + ci * kBlk;
                for (int ki = 0; ki < kBlk; ++ki) {
                    const float gv = gp[ki];
                    if (SPARSE && !(gv != 0.f)) continue;
                    acc = fmaf(gv, wp[ki], acc);
                }
            }
        }
    }
    if (active) dx[act_off(n, cb, ih, iw, CB, d.H, d.W) + ci] = acc;
}

// dw[k,c,v,u] for k = 64*blockIdx.y + lane, (c,v,u) from blockIdx.x
template <bool SPARSE>
__global__ __launch_bounds__(64) void generic_bww_kernel(st_conv_desc d, int OH, int OW,
                                                         const float *__restrict__ x,
                                                         const float *__restrict__ dy,
                                                         float *__restrict__ dw, const unsigned *sel)
{
    if (deselected(sel, 0)) return;
    const int lane = threadIdx.x;
    const int k = blockIdx.y * kWave + lane;
    int t = blockIdx.x;
    const int u = t % d.R; t /= d.R;
    const int v = t % d.S; t /= d.S;
    const int c = t;
    const int CB = d.C / kBlk, KB = d.K / kBlk;
    const bool active = k < d.K;
    const int kb = active ? k / kBlk : 0, ki = k % kBlk;
    const int cb = c / kBlk, ci = c % kBlk;
    float acc = 0.f;
    for (int n = 0; n < d.N; ++n)
        for (int oh = 0; oh < OH; ++oh) {
            const int ih = oh * d.stride_h - d.pad_h + v;
            if (ih < 0 || ih >= d.H) continue;
            for (int ow = 0; ow < OW; ++ow) {
                const int iw = ow * d.stride_w - d.pad_w + u;
                if (iw < 0 || iw >= d.W) continue;
                const float xv = x[act_off(n, cb, ih, iw, CB, d.H, d.W) + ci];
                if (SPARSE && !(xv != 0.f)) continue;
                acc = fmaf(xv, dy[act_off(n, kb, oh, ow, KB, OH, OW) + ki], acc);
            }
        }
    if (active) dw[flt_off(kb, cb, v, u, CB, d.S, d.R) + ci * kBlk + ki] = acc;
}

// dw[k,c,v,u] for c = 64*blockIdx.y + lane, (k,v,u) from blockIdx.x; the tested operand is dy
__global__ __launch_bounds__(64) void generic_bww_dy_kernel(st_conv_desc d, int OH, int OW,
                                                            const float *__restrict__ x,
                                                            const float *__restrict__ dy,
                                                            float *__restrict__ dw, const unsigned *sel)
{
    if (deselected(sel, 1)) return;
    const int lane = threadIdx.x;
    const int c = blockIdx.y * kWave + lane;
    int t = blockIdx.x;
    const int u = t % d.R; t /= d.R;
    const int v = t % d.S; t /= d.S;
    const int k = t;
    const int CB = d.C / kBlk, KB = d.K / kBlk;
    const bool active = c < d.C;
    const int cb = active ? c / kBlk : 0, ci = c % kBlk;
    const int kb = k / kBlk, ki = k % kBlk;
    float acc = 0.f;
    for (int n = 0; n < d.N; ++n)
        for (int oh = 0; oh < OH; ++oh) {
            const int ih = oh * d.stride_h - d.pad_h + v;
            if (ih < 0 || ih >= d.H) continue;
            for (int ow = 0; ow < OW; ++ow) {
                const int iw = ow * d.stride_w - d.pad_w + u;
                if (iw < 0 || iw >= d.W) continue;
                const float gv = dy[act_off(n, kb, oh, ow, KB, OH, OW) + ki];     // same address in every lane
                if (!(gv != 0.f)) continue;
                acc = fmaf(x[act_off(n, cb, ih, iw, CB, d.H, d.W) + ci], gv, acc);
            }
        }
    if (active) dw[flt_off(kb, cb, v, u, CB, d.S, d.R) + ci * kBlk + ki] = acc;
}

// Zero statistics for the choice of the form (SparseTrain Sec. 5.3 picks per layer the operand with the higher
// average sparsity and combines the kernels with dense ones): one workgroup per tensor counts the zeros of a
// sample: four workgroups per tensor (zero_sample_block) write their {zeros, elements looked at} pairs, word
// kSelThr receives the dense threshold of st_conv_bww_auto.  Nothing is accumulated, so nothing has to be
// cleared first and a single launch does it.
__global__ __launch_bounds__(256) void zero_sample_kernel(const float *__restrict__ x, size_t nx,
                                                          const float *__restrict__ dy, size_t ny,
                                                          unsigned *__restrict__ out, unsigned dense_thr)
{
    __shared__ unsigned red[8];
    const int part = blockIdx.x % kSampleParts;
    if (blockIdx.x < kSampleParts) {
        zero_sample_block(x, nx, part, out, red);
        if (blockIdx.x == 0 && threadIdx.x == 0) out[kSelThr] = dense_thr;
    } else {
        zero_sample_block(dy, ny, part, out + kSelDy, red);
    }
}

// Everything st_conv_fwd_auto / st_conv_bwi_auto need before their two main kernels, in one launch:
// the first four workgroups sample the tested operand, the next n_wave workgroups write the filter copy of the zero-skipping
// form, the rest the filter copy of the dense form.  The copies cannot know the sample's verdict (same launch),
// so both are written: at most 2 x 9.4 MB on the layers of the paper's Table 1, against one launch and its
// gap saved twice.
struct PrepareArgs {
    const float *act;           // tested operand
    size_t n_act;
    const float *w;             // the layer's filters, library layout
    float *wl, *wd;             // the two copies
    unsigned *sel;              // counters
    int KB, CB, S, R;           // filter blocks of the layer
    int Ko, Ci;                 // produced / reduced channels of the correlation the kernels run
    int transpose;              // BWI
    int paired;                 // layout of the first copy (fwd_sparse_filters_paired)
    unsigned n_wave;            // workgroups of the first copy
    size_t total_dense;         // elements of the second copy
};

__global__ __launch_bounds__(256) void auto_prepare_kernel(PrepareArgs a)
{
    __shared__ float tile[2 * kBlk][kBlk + 1];
    __shared__ unsigned red[8];
    const unsigned b = blockIdx.x;
    if (b < kSampleParts) {
        zero_sample_block(a.act, a.n_act, (int)b, a.sel, red);
    } else if (b < kSampleParts + a.n_wave) {
        if (a.transpose) wave_filters_block<true>((int)(b - kSampleParts), a.KB, a.CB, a.S, a.R, a.w, a.wl, tile, a.paired);
        else wave_filters_block<false>((int)(b - kSampleParts), a.KB, a.CB, a.S, a.R, a.w, a.wl, tile, a.paired);
    } else {
        reformat_filters_block(b - kSampleParts - a.n_wave, a.Ko, a.Ci, a.S, a.R, a.transpose, a.w, a.wd, a.total_dense);
    }
}

inline void out_dims(const st_conv_desc &d, int &OH, int &OW)
{
    OH = (d.H + 2 * d.pad_h - d.S) / d.stride_h + 1;
    OW = (d.W + 2 * d.pad_w - d.R) / d.stride_w + 1;
}

}  // namespace

hipError_t launch_generic_fwd(const st_conv_desc &d, const float *x, const float *w, float *y,
                              bool sparse, hipStream_t s, const unsigned *sel, unsigned thr)
{
    int OH, OW;
    out_dims(d, OH, OW);
    dim3 grid(OH * OW, ceil_div(d.K, kWave), d.N);
    if (sparse)
        hipLaunchKernelGGL(generic_fwd_kernel<true>, grid, dim3(64), 0, s, d, OH, OW, x, w, y, sel, thr);
    else
        hipLaunchKernelGGL(generic_fwd_kernel<false>, grid, dim3(64), 0, s, d, OH, OW, x, w, y, sel, thr);
    return hipGetLastError();
}

hipError_t launch_generic_bwi(const st_conv_desc &d, const float *dy, const float *w, float *dx,
                              bool sparse, hipStream_t s, const unsigned *sel, unsigned thr)
{
    int OH, OW;
    out_dims(d, OH, OW);
    dim3 grid(d.H * d.W, ceil_div(d.C, kWave), d.N);
    if (sparse)
        hipLaunchKernelGGL(generic_bwi_kernel<true>, grid, dim3(64), 0, s, d, OH, OW, dy, w, dx, sel, thr);
    else
        hipLaunchKernelGGL(generic_bwi_kernel<false>, grid, dim3(64), 0, s, d, OH, OW, dy, w, dx, sel, thr);
    return hipGetLastError();
}

hipError_t launch_generic_bww(const st_conv_desc &d, const float *x, const float *dy, float *dw,
                              bool sparse, hipStream_t s, const unsigned *sel)
{
    int OH, OW;
    out_dims(d, OH, OW);
    dim3 grid(d.C * d.S * d.R, ceil_div(d.K, kWave), 1);
    if (sparse)
        hipLaunchKernelGGL(generic_bww_kernel<true>, grid, dim3(64), 0, s, d, OH, OW, x, dy, dw, sel);
    else
        hipLaunchKernelGGL(generic_bww_kernel<false>, grid, dim3(64), 0, s, d, OH, OW, x, dy, dw, sel);
    return hipGetLastError();
}

hipError_t launch_generic_bww_dy(const st_conv_desc &d, const float *x, const float *dy, float *dw,
                                 hipStream_t s, const unsigned *sel)
{
    int OH, OW;
    out_dims(d, OH, OW);
    dim3 grid(d.K * d.S * d.R, ceil_div(d.C, kWave), 1);
    hipLaunchKernelGGL(generic_bww_dy_kernel, grid, dim3(64), 0, s, d, OH, OW, x, dy, dw, sel);
    return hipGetLastError();
}

hipError_t launch_zero_sample(const float *x, size_t nx, const float *dy, size_t ny, unsigned *counters,
                              hipStream_t s, unsigned dense_thr)
{
    hipLaunchKernelGGL(zero_sample_kernel, dim3(dy ? 2 * kSampleParts : kSampleParts), dim3(256), 0, s, x, nx, dy, ny, counters,
                       dense_thr);
    return hipGetLastError();
}

hipError_t launch_auto_prepare(const Geom &g, bool transpose, const float *act, size_t n_act, const float *w,
                               float *wl, float *wd, unsigned *sel, hipStream_t s)
{
    PrepareArgs a;
    a.act = act; a.n_act = n_act; a.w = w; a.wl = wl; a.wd = wd; a.sel = sel;
    a.KB = (transpose ? g.Ci : g.Ko) / kBlk; a.CB = (transpose ? g.Ko : g.Ci) / kBlk;       // of the layer
    a.S = g.S; a.R = g.R; a.Ko = g.Ko; a.Ci = g.Ci; a.transpose = transpose ? 1 : 0;
    a.paired = fwd_sparse_filters_paired(g) ? 1 : 0;
    const long long n_wave = (long long)a.KB * a.CB * g.S * g.R;
    a.total_dense = fwd_dense_filter_bytes(g) / sizeof(float);
    const long long n_dense = (long long)((a.total_dense + 255) / 256);
    if (n_wave + n_dense + kSampleParts > 0x7fffffffLL) return hipErrorInvalidValue;
    a.n_wave = (unsigned)n_wave;
    hipLaunchKernelGGL(auto_prepare_kernel, dim3((unsigned)(kSampleParts + n_wave + n_dense)), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace st
