// Device-side bodies shared by the stand-alone filter-copy kernels and by the one-launch preparation of the
// self-selecting entry points (st_conv_fwd_auto / st_conv_bwi_auto): the filter copy in wavefront order that
// the zero-skipping FWD/BWI kernel reads, the copy in MFMA lane order that the dense one reads, and the zero
// count of a sample of a tensor.  All three are written for workgroups of 256 threads.
#pragma once
#include "st_common.hpp"

namespace st {

#if defined(__HIPCC__)
// One 16x16 filter block (kb, cb, v, u) = `block` of the LAYER's filters w (library layout) into the
// wavefront-ordered copy wl[Ko/64][Ci][S][R][64 k] (Ko rounded up to whole groups of 64; the padding is never
// written and never used), or, with paired set, wl[Ko/128][Ci][S][R][64][2]: produced channels k and k + 64 of a
// group of 128 side by side (Ko is then a multiple of 128).  TRANSPOSE selects the BWI form (channel roles
// exchanged, taps reversed; SparseTrain Sec. 3.3).  tile: 32 x 17 floats of LDS; with TRANSPOSE every thread of
// the workgroup must make the call.
__device__ __forceinline__ size_t wave_filters_index(int ko, int ci, int tap, int Ci, int SR, int paired)
{
    if (paired) return ((size_t)(ko / 128) * Ci + ci) * (SR * 128) + tap * 128 + (ko % kWave) * 2 + (ko / kWave) % 2;
    return ((size_t)(ko / kWave) * Ci + ci) * (SR * kWave) + tap * kWave + ko % kWave;
}

template <bool TRANSPOSE>
__device__ __forceinline__ void wave_filters_block(int block, int KB, int CB, int S, int R, const float *__restrict__ w,
                                                   float *__restrict__ wl, float (*tile)[kBlk + 1], int paired)
{
    int t = block;
    const int u = t % R; t /= R;
    const int v = t % S; t /= S;
    const int cb = t % CB;
    const int kb = t / CB;
    const int a = threadIdx.x / kBlk, b = threadIdx.x % kBlk;
    const size_t blk = (size_t)S * R * (kBlk * kBlk);
    const size_t src = (((size_t)kb * CB + cb) * S + v) * R * (kBlk * kBlk) + (size_t)u * (kBlk * kBlk);     // [ci = a][ki = b]
    const int SR = S * R;
    if (paired) {
        // The block of the lower 64 channels of a group of 128 writes both partners, 8 contiguous bytes per
        // thread; the block of the upper 64 has nothing left to do (uniform: the whole workgroup leaves).
        // tile: 32 x 17 floats here.
        const int pb = TRANSPOSE ? cb : kb;             // block of the produced channel
        if (pb % 8 >= 4) return;
        const size_t src1 = src + (TRANSPOSE ? 4 * blk : 4 * (size_t)CB * blk);      // partner: cb + 4 or kb + 4
        float2 val;
        if constexpr (!TRANSPOSE) {
            const int k = kb * kBlk + b, c = cb * kBlk + a;
            val = make_float2(w[src + a * kBlk + b], w[src1 + a * kBlk + b]);
            *reinterpret_cast<float2 *>(wl + wave_filters_index(k, c, v * R + u, CB * kBlk, SR, 1)) = val;
        } else {
            tile[a][b] = w[src + a * kBlk + b];
            tile[kBlk + a][b] = w[src1 + a * kBlk + b];
            __syncthreads();
            const int c = cb * kBlk + b, k = kb * kBlk + a;
            val = make_float2(tile[b][a], tile[kBlk + b][a]);
            *reinterpret_cast<float2 *>(wl + wave_filters_index(c, k, (S - 1 - v) * R + (R - 1 - u), KB * kBlk, SR, 1)) = val;
        }
        return;
    }
    if constexpr (!TRANSPOSE) {
        const int k = kb * kBlk + b, c = cb * kBlk + a;
        wl[wave_filters_index(k, c, v * R + u, CB * kBlk, SR, 0)] = w[src + a * kBlk + b];
    } else {
        tile[a][b] = w[src + a * kBlk + b];
        __syncthreads();
        // produced channel = c (fast index b), reduced channel = k (a)
        const int c = cb * kBlk + b, k = kb * kBlk + a;
        wl[wave_filters_index(c, k, (S - 1 - v) * R + (R - 1 - u), KB * kBlk, SR, 0)] = tile[b][a];
    }
}

// Element i = 256 * block + thread of the copy in MFMA consumption order.  transpose = 0:
// B[k][c][tap] = w[k][c][tap] (FWD); transpose = 1: the roles of the channel dimensions are swapped and the
// taps reversed (BWI).  Ko/Ci are the produced and reduced channel counts of the correlation that will consume
// the copy; produced channels are padded with zeros to a multiple of 128.
__device__ __forceinline__ void reformat_filters_block(size_t block, int Ko, int Ci, int S, int R, int transpose,
                                                       const float *__restrict__ w, float *__restrict__ wd, size_t total)
{
    const size_t i = block * 256 + threadIdx.x;
    if (i >= total) return;
    const int TAPS = S * R, CiB = Ci / kBlk;
    size_t t = i;
    const int j = t % 8; t /= 8;
    const int l32 = t % 32; t /= 32;
    const int half = t % 2; t /= 2;
    const int tap = t % TAPS; t /= TAPS;
    const int cb = t % CiB;
    const int kb32 = (int)(t / CiB);
    const int ko = kb32 * 32 + l32, ci = cb * kBlk + half * 8 + j;
    float val = 0.f;
    if (ko < Ko) {
        const int v = tap / R, u = tap % R;
        if (!transpose) {
            // w[K = Ko][C = Ci]: element [ko/16][ci/16][v][u][ci%16][ko%16]
            val = w[((((size_t)(ko / kBlk) * CiB + ci / kBlk) * S + v) * R + u) * (kBlk * kBlk) + (ci % kBlk) * kBlk + ko % kBlk];
        } else {
            // w[K = Ci][C = Ko]: element [ci/16][ko/16][S-1-v][R-1-u][ko%16][ci%16]
            const int KoB = Ko / kBlk;
            val = w[((((size_t)(ci / kBlk) * KoB + ko / kBlk) * S + (S - 1 - v)) * R + (R - 1 - u)) * (kBlk * kBlk) + (ko % kBlk) * kBlk + ci % kBlk];
        }
    }
    wd[i] = val;
}

// Zero statistics of one tensor: the elements equal to zero in a sample of the tensor, one block of 1024
// consecutive floats out of every `stride` blocks, kSampleBlocks (64) blocks at most, 65 536 elements: enough to
// fix a zero fraction to 0.2 %.  kSampleParts (4) workgroups of 256 threads share the sample; part `part` looks
// at the sampled blocks part, part + 4, ... with all its 16 loads per thread in flight at once (one memory
// round trip, whatever the tensor size) and WRITES {zeros, elements looked at} to out[2 * part], out[2 * part + 1]:
// nothing is accumulated across workgroups, so no counter has to be cleared first and no atomics are involved;
// the readers add the four pairs (sample_zeros / sample_seen).  red: 8 unsigned of LDS.  Every thread of the
// workgroup must make the call.
constexpr int kSampleBlocks = 64, kSampleParts = 4;
__device__ __forceinline__ void zero_sample_block(const float *__restrict__ t, size_t n, int part, unsigned *__restrict__ out,
                                                  unsigned *red)
{
    const size_t blocks = (n + 1023) / 1024;
    const size_t stride = (blocks + kSampleBlocks - 1) / kSampleBlocks;
    const size_t sampled = (blocks + stride - 1) / stride;
    unsigned zeros = 0, seen = 0;
    constexpr int UN = kSampleBlocks / kSampleParts;
    float4 v[UN];
    bool full[UN];
#pragma unroll
    for (int i = 0; i < UN; ++i) {
        const size_t sb = (size_t)i * kSampleParts + part;
        const size_t base = sb * stride * 1024 + threadIdx.x * 4;
        full[i] = sb < sampled && base + 3 < n;             // tensors are 64-byte aligned: one 16-byte load
        v[i] = full[i] ? *reinterpret_cast<const float4 *>(t + base) : make_float4(1.f, 1.f, 1.f, 1.f);
    }
#pragma unroll
    for (int i = 0; i < UN; ++i) {
        const size_t sb = (size_t)i * kSampleParts + part;
        const size_t base = sb * stride * 1024 + threadIdx.x * 4;
        if (full[i]) {
            zeros += (v[i].x == 0.f ? 1u : 0u) + (v[i].y == 0.f ? 1u : 0u) + (v[i].z == 0.f ? 1u : 0u) + (v[i].w == 0.f ? 1u : 0u);
            seen += 4u;
        } else if (sb < sampled) {
            for (int j = 0; j < 4; ++j)
                if (base + j < n) {
                    zeros += t[base + j] == 0.f ? 1u : 0u;
                    seen += 1u;
                }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        zeros += __shfl_down(zeros, off);
        seen += __shfl_down(seen, off);
    }
    if (threadIdx.x % kWave == 0) {
        red[threadIdx.x / kWave] = zeros;
        red[4 + threadIdx.x / kWave] = seen;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        out[2 * part] = red[0] + red[1] + red[2] + red[3];
        out[2 * part + 1] = red[4] + red[5] + red[6] + red[7];
    }
}
#endif

}  // namespace st
