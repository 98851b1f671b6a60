// Shared declarations of the gfx950 convolution library (internal; the public
// interface is include/st_conv.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <type_traits>

#include "st_conv.h"

namespace st {

constexpr int kBlk = 16;        // channel block of the blocked layouts
constexpr int kWave = 64;       // CDNA wavefront width
constexpr size_t kFilterBytesTileMajor = 3u << 20;  // largest filter copy the zero-skipping FWD/BWI keeps L2-resident across channel tiles
constexpr int kMaxDevices = 64; // per-device set-up state is kept for this many devices of a process

// Geometry of one correlation "act_out[n,ko,oh,ow] = sum act_in[n,ci,oh*P-ph+v,ow*O-pw+u] * f[ko,ci,v,u]".
// FWD uses it directly; stride-1 BWI is the same correlation on dy with transposed, tap-reversed
// filters (SparseTrain Sec. 3.3), so both passes share this struct and the kernels built on it.
struct Geom {
    int N;
    int Ci, Ko;          // reduced (input) channels, produced (output) channels
    int Hi, Wi;          // spatial size of the input activation
    int Ho, Wo;          // spatial size of the output activation
    int R, S;            // filter width, height
    int sw, sh;          // strides
    int pw, ph;          // padding
    int uw, uh;          // spacing of the input samples on the grid the taps slide over (1; 2 for the
                         // BWI of a stride-2 layer, whose dy is spread out with zeros in between)
    // sparse/dense choice on the device (st_conv_fwd_auto, st_conv_bwi_auto): when sel is set the
    // launch does nothing unless the sampled zero fraction of the tested operand (sample_zeros / sample_seen of sel)
    // selects this form: the zero-skipping one (want = 0) from thr per mille upwards, else the
    // dense one (want = 1)
    const unsigned *sel;
    int want;
    unsigned thr;
    // host side only (st_conv_kernel_name): when set, the launcher of the zero-skipping kernel writes the
    // name of the kernel instance it would launch here and launches nothing
    char *describe;
    int describe_len;
};

#if defined(__HIPCC__)
typedef float floatx16 __attribute__((ext_vector_type(16)));       // accumulator block of a 32x32 MFMA

// element offset of pixel (h, w) of channel block cb of image n in the blocked activation layout
__device__ __forceinline__ size_t act_off(int n, int cb, int h, int w, int CB, int H, int W)
{
    return ((((size_t)n * CB + cb) * H + h) * W + w) * kBlk;
}

// f(integral_constant<int, I>) for I = First .. Last-1, fully unrolled with compile-time indices (what
// keeps register arrays indexed by them in registers)
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// immediate of s_waitcnt that waits until at most n vector-memory loads are outstanding and leaves
// the other counters alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
constexpr int vmcnt_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4) | (0xF << 8); }

// The zero-skipping FWD / BWI kernel with two channels per lane on unit-stride 3x3 layers keeps the two channels
// of a lane in register pairs and reads their filters from a copy with the two side by side
// (st_fwd_sparse_impl.hpp explains why); the kernel template and the host-side choice of the copy's layout
// both ask here.
constexpr bool fwd_sparse_paired(int R, int S, int KPL, int SD, int SU)
{
    return KPL == 2 && R == 3 && S == 3 && SD == 1 && SU == 1;
}

// Counters written by the sampling workgroups (zero_sample_block): four {zeros, elements} pairs per tensor,
// x (or the one tested operand) in words 0..7, dy in words 8..15, the dense threshold of st_conv_bww_auto in
// word 16.
constexpr int kSelDy = 8, kSelThr = 16;
__device__ __forceinline__ unsigned sample_zeros(const unsigned *c) { return c[0] + c[2] + c[4] + c[6]; }
__device__ __forceinline__ unsigned sample_seen(const unsigned *c) { return c[1] + c[3] + c[5] + c[7]; }

__device__ __forceinline__ bool form_deselected(const unsigned *sel, int want, unsigned thr)
{
    if (!sel) return false;
    const bool sparse = (unsigned long long)sample_zeros(sel) * 1000ull >= (unsigned long long)thr * sample_seen(sel);
    return (sparse ? 0 : 1) != want;
}

// BWW form choice (st_conv_bww_auto).  dy (form 1) is tested when its zero fraction exceeds that of x by
// more than 3 percentage points, else x (form 0): at equal zero fractions the form that tests dy is the
// slower one by 1-15 % (it writes its partial sums transposed), so a tie in the samples must not pick it.
// When even the sparser operand has fewer zeros than the threshold, the dense form (form 2) runs instead
// (threshold 0: never)
__device__ __forceinline__ int selected_form(const unsigned *sel)
{
    const unsigned zx = sample_zeros(sel), nx = sample_seen(sel), zy = sample_zeros(sel + kSelDy), ny = sample_seen(sel + kSelDy);
    const bool dy_sparser = (unsigned long long)zy * nx * 100ull > ((unsigned long long)zx * 100ull + 3ull * nx) * ny;
    const unsigned zb = dy_sparser ? zy : zx, nb = dy_sparser ? ny : nx;
    const bool dense = (unsigned long long)zb * 1000ull < (unsigned long long)sel[kSelThr] * nb;
    return dense ? 2 : (dy_sparser ? 1 : 0);
}

__device__ __forceinline__ bool deselected(const unsigned *sel, int want)
{
    return sel && selected_form(sel) != want;
}
#endif

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ---- launchers (each returns hipSuccess or the launch error) -------------------------------
// generic kernels: any geometry the API accepts
hipError_t launch_generic_fwd(const st_conv_desc &d, const float *x, const float *w, float *y,
                              bool sparse, hipStream_t s, const unsigned *sel = nullptr, unsigned thr = 0);
hipError_t launch_generic_bwi(const st_conv_desc &d, const float *dy, const float *w, float *dx,
                              bool sparse, hipStream_t s, const unsigned *sel = nullptr, unsigned thr = 0);
// sel (here and below): device counters of launch_zero_sample; when set, the launch is a no-op unless
// they select the operand it tests (x unless dy has the strictly larger zero fraction)
hipError_t launch_generic_bww(const st_conv_desc &d, const float *x, const float *dy, float *dw,
                              bool sparse, hipStream_t s, const unsigned *sel = nullptr);
hipError_t launch_generic_bww_dy(const st_conv_desc &d, const float *x, const float *dy, float *dw,
                                 hipStream_t s, const unsigned *sel = nullptr);
// counters = zero counts of a sample of x and (unless null) of dy, at most 64 evenly spaced blocks of 1024 elements
// each, plus dense_thr, the per-mille zero fraction below which st_conv_bww_auto runs its dense form (layout:
// kSelDy, kSelThr above)
hipError_t launch_zero_sample(const float *x, size_t nx, const float *dy, size_t ny, unsigned *counters,
                              hipStream_t s, unsigned dense_thr = 0);
// one launch for st_conv_fwd_auto / st_conv_bwi_auto: sample of the tested operand into sel[0..7], the filter copy
// of the zero-skipping form into wl and that of the dense form into wd (g = the correlation the kernels run)
hipError_t launch_auto_prepare(const Geom &g, bool transpose, const float *act, size_t n_act, const float *w,
                               float *wl, float *wd, unsigned *sel, hipStream_t s);
// one main launch that runs whichever of the two forms the sample in g.sel selects (unit-stride 3x3 layers
// whose two forms both run in workgroups of four wavefronts); wl / wd = the two filter copies
bool fwd_auto_combined_supported(const Geom &g);
hipError_t launch_fwd_auto_combined(const Geom &g, const float *in, const float *wl, const float *wd, float *out, hipStream_t s);
void fwd_auto_kernel_name(const Geom &g, char *buf, size_t len);      // requires fwd_auto_combined_supported(g)
// zero fraction (per mille) of the tested operand from which the zero-skipping FWD/BWI form beats the
// dense one for this geometry (measured; 1001 = never)
unsigned fwd_sparse_threshold(const Geom &g);

// unit-stride fast paths
bool fwd_sparse_supported(const Geom &g);
// the zero-skipping kernel reads filters from a copy in wavefront order (fwd_sparse_filter_bytes)
// written by launch_wave_filters from the layer's filters w; transpose selects the BWI form (channel
// roles swapped, taps reversed); g is the geometry of the correlation the kernel runs
size_t fwd_sparse_filter_bytes(const Geom &g);
hipError_t launch_wave_filters(const Geom &g, bool transpose, const float *w, float *wl, hipStream_t s);
// whether the kernel launch_fwd_sparse picks for g reads the copy with channel pairs side by side
bool fwd_sparse_filters_paired(const Geom &g);
hipError_t launch_fwd_sparse(const Geom &g, const float *in, const float *wl, float *out, hipStream_t s);
bool fwd_dense_supported(const Geom &g);
// the dense kernel reads filters from a reformatted copy (fwd_dense_filter_bytes) written by
// launch_reformat_filters; transpose selects the BWI form (channel roles swapped, taps reversed)
size_t fwd_dense_filter_bytes(const Geom &g);
// whole workspace of the dense form: the filter copy, then the partial outputs of launches whose
// reduction is split over workgroups (few pixel tiles)
size_t fwd_dense_workspace_bytes(const Geom &g);
hipError_t launch_reformat_filters(const Geom &g, bool transpose, const float *w, float *wd, hipStream_t s);
hipError_t launch_fwd_dense(const Geom &g, const float *in, const float *wd, float *out, hipStream_t s);
// 1x1 layers with small filter matrices: whole filter in LDS, read from the library layout (no copy
// in the workspace needed); transpose selects the BWI form
bool pw_dense_direct_supported(const Geom &g);
hipError_t launch_pw_dense_direct(const Geom &g, bool transpose, const float *in, const float *w, float *out,
                                  hipStream_t s);
// 1x1 layers: matrix product per pixel, no LDS (called by launch_fwd_dense)
hipError_t launch_pw_dense(const Geom &g, const float *in, const float *wd, float *out, hipStream_t s);

bool bww_fast_supported(const st_conv_desc &d);
size_t bww_sparse_workspace(const st_conv_desc &d);
hipError_t launch_bww_sparse(const st_conv_desc &d, const float *x, const float *dy, float *dw,
                             float *ws, hipStream_t s, const unsigned *sel = nullptr);
void bww_sparse_kernel_name(const st_conv_desc &d, char *buf, size_t len);
// BWW that tests dy instead of x (operand roles exchanged, transposing final sum)
bool bww_dy_fast_supported(const st_conv_desc &d);
size_t bww_sparse_dy_workspace(const st_conv_desc &d);
hipError_t launch_bww_sparse_dy(const st_conv_desc &d, const float *x, const float *dy, float *dw,
                                float *ws, hipStream_t s, const unsigned *sel = nullptr);
size_t bww_dense_workspace(const st_conv_desc &d);
// st_conv_bww_auto in three launches (zero-skipping with either operand tested, dense, sum of the partials):
// unit-stride 3x3 layers; ws holds max(splits) * K*C*S*R floats, at least one set
bool bww_auto_merged_supported(const st_conv_desc &d);
hipError_t launch_bww_auto_merged(const st_conv_desc &d, const float *x, const float *dy, float *dw, float *ws,
                                  hipStream_t s, const unsigned *sel);
hipError_t launch_bww_dense(const st_conv_desc &d, const float *x, const float *dy, float *dw,
                            float *ws, hipStream_t s, const unsigned *sel = nullptr);
// zero fraction (per mille) of the sparser operand below which the dense BWW beats both zero-skipping forms
unsigned bww_sparse_threshold(const st_conv_desc &d);

}  // namespace st
