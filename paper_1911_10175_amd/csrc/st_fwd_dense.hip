// Dense unit-stride correlation on the matrix cores: the control the zero-skipping kernels are
// measured against (the role the library's dense "direct" convolution plays in SparseTrain
// Sec. 4).  Used for FWD and, with transposed filters, for BWI.
//
// Implicit GEMM with v_mfma_f32_32x32x2_f32: rows = 32 output pixels, columns = 32 output
// channels, reduction = 2 input channels of one filter tap per instruction.  A wavefront owns an
// 8x8 pixel tile times 32 output channels (two accumulator blocks).  The 4 wavefronts of a
// workgroup cover KQ column blocks of 4/KQ pixel tiles; the wavefronts that share a pixel tile
// stage its input halo for one 16-channel block cooperatively in LDS (zero padding is applied
// there once), double-buffered: the global loads for block cb+1 are issued at the first tap of
// block cb and written to the other buffer after the last tap, one barrier per block.  For every
// tap the A operand is read from LDS at the shifted pixel.  The B operand (filters) is read from
// a copy that a small prologue kernel writes into the workspace in the order the MFMA lanes
// consume it, [K/32][C/16][tap][c half][32 k][8 c]: a lane fetches its 8 values of a step with
// two 16-byte loads and a wavefront reads 2 KB contiguously (fetching them element-wise from the
// library layout takes 8 load instructions per 16 MFMAs and holds the matrix pipe at about half
// rate); the loads for step s+1 are in flight during the MFMAs of step s.  No tests, no skipping.
#include <cstdlib>

#include "st_common.hpp"
#include "st_filter_copies.hpp"
#include "st_fwd_dense_impl.hpp"

namespace st {
namespace {

// Prologue: filters in MFMA consumption order (st_filter_copies.hpp).
__global__ __launch_bounds__(256) void reformat_filters_kernel(int Ko, int Ci, int S, int R, int transpose,
                                                               const float *__restrict__ w,
                                                               float *__restrict__ wd, size_t total,
                                                               const unsigned *sel, unsigned thr)
{
    if (form_deselected(sel, 1, thr)) return;       // the copy of a form that will not run is not written
    reformat_filters_block(blockIdx.x, Ko, Ci, S, R, transpose, w, wd, total);
}

// out = part[0] + part[1] + ... (fixed order), float4 at a time, on a capped grid
__global__ __launch_bounds__(256) void sum_partials_kernel(const float4 *__restrict__ part, float4 *__restrict__ out,
                                                           size_t n4, int splits, const unsigned *sel, unsigned thr)
{
    if (form_deselected(sel, 1, thr)) return;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
        float4 a = part[i];
        for (int p = 1; p < splits; ++p) {
            const float4 v = part[(size_t)p * n4 + i];
            a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
        }
        out[i] = a;
    }
}

template <int R, int S, int KQ, int TWD, int MODE = 0, int PI = 0, int PJ = 0>
hipError_t launch_cfg(const Geom &g, const float *in, const float *wd, float *out, hipStream_t s)
{
    using Cfg = FwdDenseCfg<R, S, TWD, MODE, PI, PJ>;
    constexpr int TQ = 4 / KQ;
    // MODE 2 tiles the positions of one parity class: (Ho - PI + 1) / 2 rows, (Wo - PJ + 1) / 2 columns
    const int rows = MODE == 2 ? (g.Ho - PI + 1) / 2 : g.Ho, cols = MODE == 2 ? (g.Wo - PJ + 1) / 2 : g.Wo;
    if (rows <= 0 || cols <= 0) return hipSuccess;
    const int tiles_w = ceil_div(cols, Cfg::TW), tiles_h = ceil_div(rows, Cfg::TH);
    const long long total_tiles = (long long)tiles_w * tiles_h * g.N;
    const int kgroups = ceil_div(g.Ko, 32 * KQ);
    const long long blocks = (total_tiles + TQ - 1) / TQ * kgroups;
    if (total_tiles > 0x7fffffffLL || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const int cs = MODE == 0 ? dense_channel_split(g) : 1;
    const size_t n_out = (size_t)g.N * g.Ko * g.Ho * g.Wo;
    // partial outputs sit behind the filter copy in the workspace
    float *part = cs > 1 ? const_cast<float *>(wd) + (fwd_dense_filter_bytes(g) + 255) / 256 * 256 / sizeof(float) : out;
    hipLaunchKernelGGL((fwd_dense_kernel<R, S, KQ, TWD, MODE, PI, PJ>), dim3((unsigned)blocks, cs), dim3(256), 0, s, g, in, wd,
                       part, tiles_w, tiles_h, kgroups, (int)total_tiles, cs, n_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || cs == 1) return e;
    const size_t n4 = n_out / 4;
    hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)(n4 / 256 + 1 < 1024 ? n4 / 256 + 1 : 1024)), dim3(256), 0, s,
                       reinterpret_cast<const float4 *>(part), reinterpret_cast<float4 *>(out), n4, cs, g.sel, g.thr);
    return hipGetLastError();
}

template <int R, int S, int TWD, int MODE = 0, int PI = 0, int PJ = 0>
hipError_t launch_kq(const Geom &g, const float *in, const float *wd, float *out, hipStream_t s)
{
    // the stride-2 halo is four times larger: one pixel tile per workgroup is all that fits in LDS
    // (with at most 64 output channels some of its four wavefronts then only help staging)
    if constexpr (MODE == 1) {
        return launch_cfg<R, S, 4, TWD, MODE, PI, PJ>(g, in, wd, out, s);
    } else {
        if (g.Ko > 64) return launch_cfg<R, S, 4, TWD, MODE, PI, PJ>(g, in, wd, out, s);
        if (g.Ko > 32) return launch_cfg<R, S, 2, TWD, MODE, PI, PJ>(g, in, wd, out, s);
        return launch_cfg<R, S, 1, TWD, MODE, PI, PJ>(g, in, wd, out, s);
    }
}

// stride-2 FWD: 8x8 output tiles (17x17 input halo), 4x14 tiles (9x29) for 14-wide outputs
hipError_t launch_s2_fwd(const Geom &g, const float *in, const float *wd, float *out, hipStream_t s)
{
    if (g.Wo % 8 != 0 && g.Wo % 14 == 0 && g.Ho % 4 <= g.Ho % 8) return launch_kq<3, 3, 14, 1>(g, in, wd, out, s);
    return launch_kq<3, 3, 8, 1>(g, in, wd, out, s);
}

// BWI of a stride-2 layer: the four parity classes of the dx positions, one launch each
template <int TWD>
hipError_t launch_s2_bwi_tw(const Geom &g, const float *in, const float *wd, float *out, hipStream_t s)
{
    hipError_t e = launch_kq<3, 3, TWD, 2, 1, 1>(g, in, wd, out, s);        // 4 taps: the longest first
    if (e == hipSuccess) e = launch_kq<3, 3, TWD, 2, 1, 0>(g, in, wd, out, s);
    if (e == hipSuccess) e = launch_kq<3, 3, TWD, 2, 0, 1>(g, in, wd, out, s);
    if (e == hipSuccess) e = launch_kq<3, 3, TWD, 2, 0, 0>(g, in, wd, out, s);
    return e;
}

hipError_t launch_s2_bwi(const Geom &g, const float *in, const float *wd, float *out, hipStream_t s)
{
    const int cols = g.Wo / 2;                      // columns of a parity class (up to one more for PJ = 0)
    if (cols % 8 != 0 && cols % 14 == 0) return launch_s2_bwi_tw<14>(g, in, wd, out, s);
    return launch_s2_bwi_tw<8>(g, in, wd, out, s);
}

template <int R, int S>
hipError_t launch_rs(const Geom &g, const float *in, const float *wd, float *out, hipStream_t s)
{
    int twd, kq;
    long long blocks;
    dense_tiling(g, &twd, &kq, &blocks);
    if (twd == 28) return launch_kq<R, S, 28>(g, in, wd, out, s);
    if (twd == 14) return launch_kq<R, S, 14>(g, in, wd, out, s);
    return launch_kq<R, S, 8>(g, in, wd, out, s);
}

}  // namespace

bool fwd_dense_supported(const Geom &g)
{
    if (g.sw != g.sh || g.uw != g.uh) return false;
    if (g.sw == 2 && g.uw == 1) return g.R == 3 && g.S == 3 && g.pw <= 2 && g.ph <= 2;
    if (g.sw == 1 && g.uw == 2) return g.R == 3 && g.S == 3 && g.pw == 1 && g.ph == 1;
    if (g.sw != 1 || g.uw != 1) return false;
    if (g.R == 3 && g.S == 3) return g.pw <= 2 && g.ph <= 2;
    if (g.R == 1 && g.S == 1) return g.pw == 0 && g.ph == 0;
    return false;
}

size_t fwd_dense_filter_bytes(const Geom &g)
{
    // output channels padded to a multiple of 128 so that every column block a workgroup touches exists
    return (size_t)ceil_div(g.Ko, 128) * 128 * g.Ci * g.S * g.R * sizeof(float);
}

size_t fwd_dense_workspace_bytes(const Geom &g)
{
    // filter copy, then the partial outputs of a channel-split launch
    const size_t n = fwd_dense_filter_bytes(g);
    const int cs = dense_channel_split(g);
    if (cs == 1) return n;
    return (n + 255) / 256 * 256 + (size_t)cs * g.N * g.Ko * g.Ho * g.Wo * sizeof(float);
}

hipError_t launch_reformat_filters(const Geom &g, bool transpose, const float *w, float *wd, hipStream_t s)
{
    const size_t total = fwd_dense_filter_bytes(g) / sizeof(float);
    hipLaunchKernelGGL(reformat_filters_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, g.Ko, g.Ci,
                       g.S, g.R, transpose ? 1 : 0, w, wd, total, g.sel, g.thr);
    return hipGetLastError();
}

hipError_t launch_fwd_dense(const Geom &g, const float *in, const float *wd, float *out, hipStream_t s)
{
    if (g.sw == 2) return launch_s2_fwd(g, in, wd, out, s);
    if (g.uw == 2) return launch_s2_bwi(g, in, wd, out, s);
    if (g.R == 3 && g.S == 3) return launch_rs<3, 3>(g, in, wd, out, s);
    if (g.R == 1 && g.S == 1) {
        // minibatch-wide pixel numbering of the pointwise kernel is kept in int
        if ((long long)g.N * g.Ho * g.Wo <= 0x7fffff00LL) return launch_pw_dense(g, in, wd, out, s);
        return launch_rs<1, 1>(g, in, wd, out, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace st
