// Zero-skipping correlation for FWD and (with transposed filters) BWI: geometry checks, the filter
// copy in wavefront order and the choice of the kernel shape.  The kernel template is in
// st_fwd_sparse_impl.hpp; its instances are compiled in the st_fwd_sparse_*.hip files (one per family,
// so that they build in parallel).
#include "st_common.hpp"
#include "st_filter_copies.hpp"

namespace st {

namespace fs {
// 3x3, unit stride: 128 or 64 produced channels per wavefront
hipError_t launch_s1_k2(const Geom &g, const float *in, const float *f, float *out, hipStream_t s);
hipError_t launch_s1_k1(const Geom &g, const float *in, const float *f, float *out, hipStream_t s);
// 3x3 of a stride-2 layer: FWD (output samples every second position) and BWI (input samples on every second position)
hipError_t launch_s2_fwd(const Geom &g, const float *in, const float *f, float *out, hipStream_t s);
hipError_t launch_s2_bwi(const Geom &g, const float *in, const float *f, float *out, hipStream_t s);
// 1x1
hipError_t launch_pw(const Geom &g, const float *in, const float *f, float *out, hipStream_t s);
}  // namespace fs

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
// with 128 output channels per wavefront and 36-41 % with 64; the stride-2 FWD tests 2.25 taps
// per element and its BWI is held by the filter stream of small tiles; a 1x1 layer saves K/64
// multiply-adds per zero.
unsigned fwd_sparse_threshold(const Geom &g)
{
    if (!fwd_sparse_supported(g)) return 0;         // generic kernels: the test only ever removes work
    if (g.R == 1) return 1001;          // 1x1: at most K/64 multiply-adds per test, behind the matrix cores even at 95 % zeros
    if (g.sw == 2) return 800;
    if (g.uw == 2) return 450;
    const bool wide = g.Ko % 128 == 0;
    return wide ? 250 : 400;
}

namespace {

// Filters in the order the wavefronts read them (st_filter_copies.hpp): one load instruction of a wavefront
// then covers 256 contiguous bytes instead of four 64-byte pieces of four cache lines, and the nine taps of a
// channel sit at immediate offsets of one address.  KB x CB are the filter blocks of the LAYER.
template <bool TRANSPOSE>
__global__ __launch_bounds__(256) void wave_filters_kernel(int KB, int CB, int S, int R,
                                                           const float *__restrict__ w, float *__restrict__ wl,
                                                           const unsigned *sel, unsigned thr, int paired)
{
    if (form_deselected(sel, 0, thr)) return;       // the copy of a form that will not run is not written
    __shared__ float tile[2 * kBlk][kBlk + 1];
    wave_filters_block<TRANSPOSE>((int)blockIdx.x, KB, CB, S, R, w, wl, tile, paired);
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
    const int paired = fwd_sparse_filters_paired(g) ? 1 : 0;
    if (transpose)
        hipLaunchKernelGGL(wave_filters_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, KB, CB, g.S, g.R, w, wl, g.sel, g.thr,
                           paired);
    else
        hipLaunchKernelGGL(wave_filters_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, KB, CB, g.S, g.R, w, wl, g.sel, g.thr,
                           paired);
    return hipGetLastError();
}

// the geometries launch_fwd_sparse hands to launch_s1_k2: two channels per lane, unit-stride 3x3
bool fwd_sparse_filters_paired(const Geom &g)
{
    return g.sw == 1 && g.uw == 1 && g.R == 3 && g.S == 3 && g.Ko % 128 == 0 && fwd_sparse_paired(g.R, g.S, 2, 1, 1);
}

hipError_t launch_fwd_sparse(const Geom &g, const float *in, const float *f, float *out, hipStream_t s)
{
    if (g.sw == 2) return fs::launch_s2_fwd(g, in, f, out, s);
    if (g.uw == 2) return fs::launch_s2_bwi(g, in, f, out, s);
    if (g.R == 3 && g.S == 3) {
        if (g.Ko % 128 == 0) return fs::launch_s1_k2(g, in, f, out, s);
        return fs::launch_s1_k1(g, in, f, out, s);
    }
    if (g.R == 1 && g.S == 1) return fs::launch_pw(g, in, f, out, s);
    return hipErrorInvalidValue;
}

}  // namespace st
