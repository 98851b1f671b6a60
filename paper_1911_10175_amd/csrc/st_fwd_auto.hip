// One main launch for st_conv_fwd_auto / st_conv_bwi_auto on unit-stride 3x3 layers: the kernel holds the
// body of the zero-skipping form and the body of the dense form and runs the one the sampled zero count of
// the tested operand selects (SparseTrain Sec. 5.3 combines the two kinds of kernel per layer; here per
// call, on the device, with no empty launch for the form that does not run).  The grid is the larger of
// the two forms' grids; workgroups beyond the selected form's own leave at once.  Both bodies use the
// same 256 threads and the same LDS allocation, and compute exactly what the separate kernels compute,
// in the same order: the result is bit-identical to the direct call of the selected form.
#include <cstdio>

#include "st_fwd_dense_impl.hpp"
#include "st_fwd_sparse_impl.hpp"

namespace st {
namespace {

struct DenseGrid {
    int tiles_w, tiles_h, kgroups, total_tiles;
    long long blocks;
};

constexpr int cmax(int a, int b) { return a > b ? a : b; }

// TH x TW pixels and KPL channels per lane, CS wavefronts per task: the zero-skipping form; KQ column blocks
// per workgroup and TWD-wide tiles: the dense form
template <int TH, int TW, int KPL, int CS, int KQ, int TWD>
__global__ __launch_bounds__(256, 4) void fwd_auto_kernel(Geom g, const float *__restrict__ in, const float *__restrict__ wl,
                                                          const float *__restrict__ wd, float *__restrict__ out,
                                                          SparseGrid sq, DenseGrid dq)
{
    static_assert(CS <= 4, "both forms run in workgroups of four wavefronts");
    __shared__ __attribute__((aligned(16))) float lds[cmax(fwd_sparse_lds_floats<3, 3, TH, TW, KPL, CS>(),
                                                           fwd_dense_lds_floats<3, 3, KQ, TWD>())];
    // uniform over the grid, before any barrier
    if (!form_deselected(g.sel, 0, g.thr)) {
        if ((long long)blockIdx.x >= sq.blocks) return;
        fwd_sparse_body<3, 3, TH, TW, KPL, CS>(g, in, wl, out, sq.tiles_w, sq.tiles_h, sq.ktiles, sq.total, sq.slots_per_xcd,
                                               sq.kt_major, lds);
    } else {
        if ((long long)blockIdx.x >= dq.blocks) return;
        fwd_dense_body<3, 3, KQ, TWD>(g, in, wd, out, dq.tiles_w, dq.tiles_h, dq.kgroups, dq.total_tiles, 1, 0, (int)blockIdx.x, 0, lds);
    }
}

template <int TH, int TW, int KPL, int CS, int KQ, int TWD>
hipError_t launch_pair(const Geom &g, const float *in, const float *wl, const float *wd, float *out, hipStream_t s)
{
    using SCfg = FwdSparseCfg<3, 3, TH, TW, KPL>;
    using DCfg = FwdDenseCfg<3, 3, TWD>;
    const SparseGrid sq = sparse_grid<TH, TW, SCfg::KT, CS>(g);
    DenseGrid dq;
    dq.tiles_w = ceil_div(g.Wo, DCfg::TW);
    dq.tiles_h = ceil_div(g.Ho, DCfg::TH);
    const long long total_tiles = (long long)dq.tiles_w * dq.tiles_h * g.N;
    dq.kgroups = ceil_div(g.Ko, 32 * KQ);
    constexpr int TQ = 4 / KQ;
    dq.blocks = (total_tiles + TQ - 1) / TQ * dq.kgroups;
    if (!sq.ok || total_tiles > 0x7fffffffLL || dq.blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    dq.total_tiles = (int)total_tiles;
    const long long blocks = sq.blocks > dq.blocks ? sq.blocks : dq.blocks;
    hipLaunchKernelGGL((fwd_auto_kernel<TH, TW, KPL, CS, KQ, TWD>), dim3((unsigned)blocks), dim3(256), 0, s, g, in, wl, wd, out, sq, dq);
    return hipGetLastError();
}

// The tile choices the separate launches make for g (launch_s1_k2 / launch_s1_k1 and launch_rs), or false
// when no combined instance exists for them
struct Pair {
    int tw, kpl, cs, kq, twd;
};

bool pick_pair(const Geom &g, Pair *p)
{
    if (g.R != 3 || g.S != 3 || g.sw != 1 || g.sh != 1 || g.uw != 1 || g.uh != 1) return false;
    if (!fwd_sparse_supported(g) || !fwd_dense_supported(g)) return false;
    if (dense_channel_split(g) != 1) return false;
    // one channel per lane (64 produced channels) is left to the separate kernels: next to the dense body it
    // loses its fifth wavefront per SIMD and runs 14-21 % slower (measured on 64->64 @224 and the BWI of 64->128 @112)
    if (g.Ko % 128 != 0) return false;
    p->kpl = 2;
    p->tw = g.Wo % 7 == 0 ? 7 : 8;                 // as launch_s1_k2
    const int th = p->kpl == 2 ? 4 : 8;
    p->cs = sparse_channel_split(g, th, p->tw, 64 * p->kpl, true);
    if (p->cs != 2 && p->cs != 4) return false;
    long long blocks;
    dense_tiling(g, &p->twd, &p->kq, &blocks);
    if (p->kq != 4) return false;
    return p->twd == 8 || (p->tw == 7 && (p->twd == 28 || p->twd == 14));
}

}  // namespace

bool fwd_auto_combined_supported(const Geom &g)
{
    Pair p;
    return pick_pair(g, &p);
}

void fwd_auto_kernel_name(const Geom &g, char *buf, size_t len)
{
    Pair p;
    if (!pick_pair(g, &p)) { if (len) buf[0] = 0; return; }
    snprintf(buf, len, "fwd_auto_kernel<%d, %d, %d, %d, %d, %d>", p.kpl == 2 ? 4 : 8, p.tw, p.kpl, p.cs, p.kq, p.twd);
}

hipError_t launch_fwd_auto_combined(const Geom &g, const float *in, const float *wl, const float *wd, float *out, hipStream_t s)
{
    Pair p;
    if (!pick_pair(g, &p)) return hipErrorInvalidValue;
    if (p.tw == 8) {
        if (p.cs == 2) return launch_pair<4, 8, 2, 2, 4, 8>(g, in, wl, wd, out, s);
        return launch_pair<4, 8, 2, 4, 4, 8>(g, in, wl, wd, out, s);
    }
    if (p.twd == 8) {
        if (p.cs == 2) return launch_pair<4, 7, 2, 2, 4, 8>(g, in, wl, wd, out, s);
        return launch_pair<4, 7, 2, 4, 4, 8>(g, in, wl, wd, out, s);
    }
    if (p.twd == 28) {
        if (p.cs == 2) return launch_pair<4, 7, 2, 2, 4, 28>(g, in, wl, wd, out, s);
        return launch_pair<4, 7, 2, 4, 4, 28>(g, in, wl, wd, out, s);
    }
    if (p.cs == 2) return launch_pair<4, 7, 2, 2, 4, 14>(g, in, wl, wd, out, s);
    return launch_pair<4, 7, 2, 4, 4, 14>(g, in, wl, wd, out, s);
}

}  // namespace st
