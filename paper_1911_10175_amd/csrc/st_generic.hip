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

struct SampleArgs {
    const float *t[2];          // x, dy (or one tensor and null)
    size_t n[2];                // elements
    unsigned stride[2];         // every stride-th block of 1024 elements is looked at
    size_t sampled[2];          // number of such blocks
};

// Zero statistics for the operand choice of BWW (SparseTrain Sec. 5.3 picks the operand with the
// higher average sparsity): counts the elements equal to zero in a sample of a tensor, one block of
// 1024 consecutive floats out of every `stride` blocks, and adds {zeros, elements looked at} to
// out[2 * tensor], out[2 * tensor + 1] with one 64-bit integer atomic per workgroup (order-independent, hence
// deterministic; the sample is capped at 2^30 elements, so the low word never carries into the high).
// Atomics to one address are serialised by the memory system at about 25 ns each: a launch uses at
// most 256 workgroups, and each keeps four loads in flight per thread instead.
// blockIdx.y selects the tensor: x and dy are sampled by one launch.
__global__ __launch_bounds__(256) void zero_sample_kernel(SampleArgs a, unsigned *__restrict__ out)
{
    __shared__ unsigned wz[4], wn[4];
    const int which = blockIdx.y;
    const float *__restrict__ t = a.t[which];
    const size_t n = a.n[which], sampled_blocks = a.sampled[which];
    const unsigned stride = a.stride[which];
    unsigned zeros = 0, seen = 0;
    constexpr int UN = 4;
    for (size_t b0 = blockIdx.x; b0 < sampled_blocks; b0 += (size_t)gridDim.x * UN) {
        float4 v[UN];
        bool full[UN];
#pragma unroll
        for (int i = 0; i < UN; ++i) {
            const size_t b = b0 + (size_t)i * gridDim.x;
            const size_t base = b * stride * 1024 + threadIdx.x * 4;
            full[i] = b < sampled_blocks && base + 3 < n;      // tensors are 64-byte aligned: one 16-byte load
            v[i] = full[i] ? *reinterpret_cast<const float4 *>(t + base) : make_float4(1.f, 1.f, 1.f, 1.f);
        }
#pragma unroll
        for (int i = 0; i < UN; ++i) {
            const size_t b = b0 + (size_t)i * gridDim.x;
            const size_t base = b * stride * 1024 + threadIdx.x * 4;
            if (full[i]) {
                zeros += (v[i].x == 0.f ? 1u : 0u) + (v[i].y == 0.f ? 1u : 0u) + (v[i].z == 0.f ? 1u : 0u) + (v[i].w == 0.f ? 1u : 0u);
                seen += 4u;
            } else if (b < sampled_blocks) {
                for (int j = 0; j < 4; ++j)
                    if (base + j < n) {
                        zeros += t[base + j] == 0.f ? 1u : 0u;
                        seen += 1u;
                    }
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        zeros += __shfl_down(zeros, off);
        seen += __shfl_down(seen, off);
    }
    if (threadIdx.x % kWave == 0) {
        wz[threadIdx.x / kWave] = zeros;
        wn[threadIdx.x / kWave] = seen;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned long long z = wz[0] + wz[1] + wz[2] + wz[3], m = wn[0] + wn[1] + wn[2] + wn[3];
        if (m) atomicAdd(reinterpret_cast<unsigned long long *>(out + 2 * which), z | (m << 32));    // 8-byte aligned
    }
}

__global__ void clear_counters_kernel(unsigned *c, unsigned dense_thr)
{
    c[threadIdx.x] = threadIdx.x < 4 ? 0u : dense_thr;
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
    hipLaunchKernelGGL(clear_counters_kernel, dim3(1), dim3(5), 0, s, counters, dense_thr);
    SampleArgs a;
    const float *t[2] = {x, dy};
    const size_t n[2] = {nx, ny};
    size_t most = 1;
    for (int i = 0; i < 2; ++i) {
        a.t[i] = t[i]; a.n[i] = t[i] ? n[i] : 0; a.stride[i] = 1; a.sampled[i] = 0;
        if (!t[i]) continue;
        const size_t blocks = (n[i] + 1023) / 1024;
        // about 1024 blocks spread evenly over the tensor (all of them when there are fewer): 10^6
        // elements fix a zero fraction to a fraction of a per cent, and the pass stays a few
        // microseconds whatever the tensor size
        const size_t stride = (blocks + 1023) / 1024;
        a.stride[i] = (unsigned)stride;
        a.sampled[i] = (blocks + stride - 1) / stride;
        if (a.sampled[i] > most) most = a.sampled[i];
    }
    hipLaunchKernelGGL(zero_sample_kernel, dim3((unsigned)(most < 256 ? most : 256), dy ? 2 : 1), dim3(256), 0, s, a,
                       counters);
    return hipGetLastError();
}

}  // namespace st
