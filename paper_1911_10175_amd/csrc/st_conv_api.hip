// C ABI of the library (include/st_conv.h): argument validation and kernel selection.
// No allocation, no synchronisation, no printing happens here.
#include <mutex>

#include "st_common.hpp"

// Built-in scratch of st_conv_fwd_static (callers that cannot allocate): the filter copy in wavefront
// order that st_conv_fwd otherwise writes into the caller's workspace.  One copy per GPU the library
// runs on, held until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress: kernels are given the device address obtained from it, never the name.
constexpr size_t kStaticScratchBytes = 16u << 20;
static __device__ __align__(256) float scratch[kStaticScratchBytes / sizeof(float)];

namespace {

using st::Geom;

struct Dims {
    int OH, OW;
};

st_status validate(const st_conv_desc *d, Dims *o)
{
    if (!d) return ST_ERR_NULL;
    if (d->N <= 0 || d->C <= 0 || d->K <= 0 || d->H <= 0 || d->W <= 0) return ST_ERR_BAD_SHAPE;
    if (d->R <= 0 || d->S <= 0 || d->stride_w <= 0 || d->stride_h <= 0) return ST_ERR_BAD_SHAPE;
    if (d->pad_w < 0 || d->pad_h < 0) return ST_ERR_BAD_SHAPE;
    if (d->C % st::kBlk || d->K % st::kBlk) return ST_ERR_BAD_SHAPE;
    if (d->H + 2 * d->pad_h < d->S || d->W + 2 * d->pad_w < d->R) return ST_ERR_BAD_SHAPE;
    o->OH = (d->H + 2 * d->pad_h - d->S) / d->stride_h + 1;
    o->OW = (d->W + 2 * d->pad_w - d->R) / d->stride_w + 1;
    // the kernels index tensors with size_t but keep grids and offsets within one channel block of
    // one image (16 floats per pixel) in int
    const long long lim = 0x7fffffffLL;
    if ((long long)d->H * d->W * st::kBlk > lim || (long long)o->OH * o->OW * st::kBlk > lim) return ST_ERR_UNSUPPORTED;
    if ((long long)d->C * d->S * d->R > lim || d->N > 65535) return ST_ERR_UNSUPPORTED;
    // padding at least as large as the filter would make whole output rows read only zeros;
    // legal, handled by the generic kernels
    return ST_OK;
}

Geom fwd_geom(const st_conv_desc &d, const Dims &o)
{
    Geom g;
    g.N = d.N; g.Ci = d.C; g.Ko = d.K;
    g.Hi = d.H; g.Wi = d.W; g.Ho = o.OH; g.Wo = o.OW;
    g.R = d.R; g.S = d.S; g.sw = d.stride_w; g.sh = d.stride_h; g.pw = d.pad_w; g.ph = d.pad_h;
    g.uw = 1; g.uh = 1;
    g.sel = nullptr; g.want = 0; g.thr = 0;
    g.describe = nullptr; g.describe_len = 0;
    return g;
}

// BWI as a correlation of dy with transposed, tap-reversed filters (SparseTrain Sec. 3.3):
// input = dy [N][K][OH][OW], output = dx [N][C][H][W], padding S-1-pad_h / R-1-pad_w.  With a
// stride the dy samples sit stride positions apart on the grid the taps slide over
// (dx[ih] = sum_v' dyU[ih - (S-1-pad_h) + v'] w[S-1-v'] with dyU[stride*oh] = dy[oh], 0 elsewhere).
bool bwi_as_fwd(const st_conv_desc &d, const Dims &o, Geom *g)
{
    if (d.pad_w > d.R - 1 || d.pad_h > d.S - 1) return false;
    g->N = d.N; g->Ci = d.K; g->Ko = d.C;
    g->Hi = o.OH; g->Wi = o.OW; g->Ho = d.H; g->Wo = d.W;
    g->R = d.R; g->S = d.S; g->sw = 1; g->sh = 1;
    g->uw = d.stride_w; g->uh = d.stride_h;
    g->pw = d.R - 1 - d.pad_w; g->ph = d.S - 1 - d.pad_h;
    g->sel = nullptr; g->want = 0; g->thr = 0;
    g->describe = nullptr; g->describe_len = 0;
    return true;
}

// Tensor arguments: all present, each on a 64-byte boundary (one pixel's channel block; the kernels
// move them with 16-byte vector loads and stores, which fault on a misaligned address).
st_status tensors_ok(const void *a, const void *b, const void *c)
{
    if (!a || !b || !c) return ST_ERR_NULL;
    if (((uintptr_t)a | (uintptr_t)b | (uintptr_t)c) % 64 != 0) return ST_ERR_ALIGNMENT;
    return ST_OK;
}

bool ws_ok(const void *ws, size_t have, size_t need)
{
    if (need == 0) return true;
    return ws != nullptr && have >= need && ((uintptr_t)ws % 256) == 0;
}

st_status dev(hipError_t e) { return e == hipSuccess ? ST_OK : ST_ERR_DEVICE; }

constexpr size_t kCounterBytes = 256;

size_t align256(size_t n) { return (n + 255) / 256 * 256; }

size_t workspace_bytes(const st_conv_desc &d, const Dims &o, int pass, bool dense)
{
    switch (pass) {
    case ST_PASS_FWD: {
        const Geom g = fwd_geom(d, o);
        if (dense) return st::fwd_dense_supported(g) ? st::fwd_dense_workspace_bytes(g) : 0;
        return st::fwd_sparse_supported(g) ? st::fwd_sparse_filter_bytes(g) : 0;
    }
    case ST_PASS_BWI: {
        Geom g;
        if (!bwi_as_fwd(d, o, &g)) return 0;
        if (dense) return st::fwd_dense_supported(g) ? st::fwd_dense_workspace_bytes(g) : 0;
        return st::fwd_sparse_supported(g) ? st::fwd_sparse_filter_bytes(g) : 0;
    }
    case ST_PASS_BWW:
        if (!st::bww_fast_supported(d)) return 0;
        return dense ? st::bww_dense_workspace(d) : st::bww_sparse_workspace(d);
    case ST_PASS_BWW_DY:
        if (dense) return workspace_bytes(d, o, ST_PASS_BWW, true);
        return st::bww_dy_fast_supported(d) ? st::bww_sparse_dy_workspace(d) : 0;
    case ST_PASS_FWD_AUTO:
    case ST_PASS_BWI_AUTO: {
        // counters, then the workspaces of the zero-skipping and of the dense form side by side
        const int base = pass == ST_PASS_FWD_AUTO ? ST_PASS_FWD : ST_PASS_BWI;
        if (dense) return workspace_bytes(d, o, base, true);
        return kCounterBytes + align256(workspace_bytes(d, o, base, false)) + workspace_bytes(d, o, base, true);
    }
    case ST_PASS_BWW_AUTO: {
        if (dense) return workspace_bytes(d, o, ST_PASS_BWW, true);
        // 256 bytes of counters, then the partial sums of whichever form runs
        const size_t a = workspace_bytes(d, o, ST_PASS_BWW, false), b = workspace_bytes(d, o, ST_PASS_BWW_DY, false);
        const size_t c = workspace_bytes(d, o, ST_PASS_BWW, true);
        size_t m = a > b ? a : b;
        if (c > m) m = c;
        // the three-launch path stages the partial sums of every form, also a single one
        const size_t one = (size_t)d.K * d.C * d.S * d.R * sizeof(float);
        if (st::bww_auto_merged_supported(d) && m < one) m = one;
        return kCounterBytes + m;
    }
    default:
        return 0;
    }
}

st_status run_fwd(const st_conv_desc *d, const float *x, const float *w, float *y, void *ws,
                  size_t ws_bytes, void *stream, bool dense)
{
    Dims o;
    st_status rc = validate(d, &o);
    if (rc != ST_OK) return rc;
    if ((rc = tensors_ok(x, w, y)) != ST_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Geom g = fwd_geom(*d, o);
    if (dense) {
        if (!st::fwd_dense_supported(g)) return dev(st::launch_generic_fwd(*d, x, w, y, false, s));
        if (!ws_ok(ws, ws_bytes, st::fwd_dense_workspace_bytes(g))) return ST_ERR_WORKSPACE;
        if (st::pw_dense_direct_supported(g)) return dev(st::launch_pw_dense_direct(g, false, x, w, y, s));
        float *wd = static_cast<float *>(ws);
        if (st::launch_reformat_filters(g, false, w, wd, s) != hipSuccess) return ST_ERR_DEVICE;
        return dev(st::launch_fwd_dense(g, x, wd, y, s));
    }
    if (!st::fwd_sparse_supported(g)) return dev(st::launch_generic_fwd(*d, x, w, y, true, s));
    if (!ws_ok(ws, ws_bytes, st::fwd_sparse_filter_bytes(g))) return ST_ERR_WORKSPACE;
    float *wl = static_cast<float *>(ws);
    if (st::launch_wave_filters(g, false, w, wl, s) != hipSuccess) return ST_ERR_DEVICE;
    return dev(st::launch_fwd_sparse(g, x, wl, y, s));
}

st_status run_bwi(const st_conv_desc *d, const float *dy, const float *w, float *dx, void *ws,
                  size_t ws_bytes, void *stream, bool dense)
{
    Dims o;
    st_status rc = validate(d, &o);
    if (rc != ST_OK) return rc;
    if ((rc = tensors_ok(dy, w, dx)) != ST_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Geom g;
    const bool fast = bwi_as_fwd(*d, o, &g) &&
                      (dense ? st::fwd_dense_supported(g) : st::fwd_sparse_supported(g));
    if (!fast) return dev(st::launch_generic_bwi(*d, dy, w, dx, !dense, s));
    float *wt = static_cast<float *>(ws);
    if (dense) {
        if (!ws_ok(ws, ws_bytes, st::fwd_dense_workspace_bytes(g))) return ST_ERR_WORKSPACE;
        if (st::pw_dense_direct_supported(g)) return dev(st::launch_pw_dense_direct(g, true, dy, w, dx, s));
        if (st::launch_reformat_filters(g, true, w, wt, s) != hipSuccess) return ST_ERR_DEVICE;
        return dev(st::launch_fwd_dense(g, dy, wt, dx, s));
    }
    if (!ws_ok(ws, ws_bytes, st::fwd_sparse_filter_bytes(g))) return ST_ERR_WORKSPACE;
    if (st::launch_wave_filters(g, true, w, wt, s) != hipSuccess) return ST_ERR_DEVICE;
    return dev(st::launch_fwd_sparse(g, dy, wt, dx, s));
}

st_status run_bww(const st_conv_desc *d, const float *x, const float *dy, float *dw, void *ws,
                  size_t ws_bytes, void *stream, bool dense)
{
    Dims o;
    st_status rc = validate(d, &o);
    if (rc != ST_OK) return rc;
    if ((rc = tensors_ok(x, dy, dw)) != ST_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!st::bww_fast_supported(*d)) return dev(st::launch_generic_bww(*d, x, dy, dw, !dense, s));
    const size_t need = dense ? st::bww_dense_workspace(*d) : st::bww_sparse_workspace(*d);
    if (!ws_ok(ws, ws_bytes, need)) return ST_ERR_WORKSPACE;
    float *wsf = static_cast<float *>(ws);
    return dev(dense ? st::launch_bww_dense(*d, x, dy, dw, wsf, s)
                     : st::launch_bww_sparse(*d, x, dy, dw, wsf, s));
}

st_status run_bww_dy(const st_conv_desc *d, const float *x, const float *dy, float *dw, void *ws,
                     size_t ws_bytes, void *stream)
{
    Dims o;
    st_status rc = validate(d, &o);
    if (rc != ST_OK) return rc;
    if ((rc = tensors_ok(x, dy, dw)) != ST_OK) return rc;
    if ((long long)d->K * d->S * d->R > 0x7fffffffLL) return ST_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!st::bww_dy_fast_supported(*d)) return dev(st::launch_generic_bww_dy(*d, x, dy, dw, s));
    if (!ws_ok(ws, ws_bytes, st::bww_sparse_dy_workspace(*d))) return ST_ERR_WORKSPACE;
    return dev(st::launch_bww_sparse_dy(*d, x, dy, dw, static_cast<float *>(ws), s));
}

// FWD (bwi = false) or BWI with the form chosen on the device: the zeros of a sample of the tested
// operand are counted, then the zero-skipping and the dense form are both enqueued and the one the
// count does not select returns at once (the filter copies of both are written regardless: they are
// small).  SparseTrain Sec. 5.3 combines its kernels with the dense ones per layer from profiles;
// this makes the same choice per call.
st_status run_fwd_bwi_auto(const st_conv_desc *d, const float *act, const float *w, float *out, void *ws,
                           size_t ws_bytes, void *stream, bool bwi)
{
    Dims o;
    st_status rc = validate(d, &o);
    if (rc != ST_OK) return rc;
    if ((rc = tensors_ok(act, w, out)) != ST_OK) return rc;
    const int pass = bwi ? ST_PASS_BWI_AUTO : ST_PASS_FWD_AUTO, base = bwi ? ST_PASS_BWI : ST_PASS_FWD;
    if (!ws_ok(ws, ws_bytes, workspace_bytes(*d, o, pass, false))) return ST_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned *sel = static_cast<unsigned *>(ws);
    char *p = static_cast<char *>(ws) + kCounterBytes;
    float *ws_sparse = reinterpret_cast<float *>(p);
    float *ws_dense = reinterpret_cast<float *>(p + align256(workspace_bytes(*d, o, base, false)));
    const size_t n_act = bwi ? (size_t)d->N * d->K * o.OH * o.OW : (size_t)d->N * d->C * d->H * d->W;

    Geom g = fwd_geom(*d, o);
    const bool as_corr = bwi ? bwi_as_fwd(*d, o, &g) : true;
    const bool fast_sparse = as_corr && st::fwd_sparse_supported(g);
    const bool fast_dense = as_corr && st::fwd_dense_supported(g);
    g.thr = fast_sparse ? st::fwd_sparse_threshold(g) : 0;
    if (!fast_dense && fast_sparse) g.thr = 0;      // tiled zero-skipping form against a generic dense one
    // Geometries whose answer does not depend on the data (break-even at 0: always zero-skipping;
    // above 1000 per mille: never) go straight to that form: no sampling, no second form enqueued.
    if (g.thr == 0 || g.thr > 1000) {
        const bool dense = g.thr > 1000;
        const size_t off = dense ? align256(workspace_bytes(*d, o, base, false)) : 0;
        const size_t left = ws_bytes > kCounterBytes + off ? ws_bytes - kCounterBytes - off : 0;
        return bwi ? run_bwi(d, act, w, out, left ? p + off : nullptr, left, stream, dense)
                   : run_fwd(d, act, w, out, left ? p + off : nullptr, left, stream, dense);
    }
    hipError_t e;
    if (fast_sparse && fast_dense && !st::pw_dense_direct_supported(g)) {
        // both forms tiled: sample and both filter copies in one launch, then one main kernel that holds both
        // forms, or, for the shapes that have none, the two main kernels, of which the one the count does not
        // select returns at once
        if (st::launch_auto_prepare(g, bwi, act, n_act, w, ws_sparse, ws_dense, sel, s) != hipSuccess) return ST_ERR_DEVICE;
        g.sel = sel;
        g.want = 0;
        if (st::fwd_auto_combined_supported(g)) return dev(st::launch_fwd_auto_combined(g, act, ws_sparse, ws_dense, out, s));
        if (st::launch_fwd_sparse(g, act, ws_sparse, out, s) != hipSuccess) return ST_ERR_DEVICE;
        g.want = 1;
        return dev(st::launch_fwd_dense(g, act, ws_dense, out, s));
    }
    if (st::launch_zero_sample(act, n_act, nullptr, 0, sel, s) != hipSuccess) return ST_ERR_DEVICE;
    g.sel = sel;
    // zero-skipping form
    g.want = 0;
    if (fast_sparse) {
        if (st::launch_wave_filters(g, bwi, w, ws_sparse, s) != hipSuccess) return ST_ERR_DEVICE;
        e = st::launch_fwd_sparse(g, act, ws_sparse, out, s);
    } else {
        e = bwi ? st::launch_generic_bwi(*d, act, w, out, true, s, sel, g.thr)
                : st::launch_generic_fwd(*d, act, w, out, true, s, sel, g.thr);
    }
    if (e != hipSuccess) return ST_ERR_DEVICE;
    // dense form
    g.want = 1;
    if (fast_dense && st::pw_dense_direct_supported(g)) {
        e = st::launch_pw_dense_direct(g, bwi, act, w, out, s);
    } else if (fast_dense) {
        if (st::launch_reformat_filters(g, bwi, w, ws_dense, s) != hipSuccess) return ST_ERR_DEVICE;
        e = st::launch_fwd_dense(g, act, ws_dense, out, s);
    } else {
        e = bwi ? st::launch_generic_bwi(*d, act, w, out, false, s, sel, g.thr)
                : st::launch_generic_fwd(*d, act, w, out, false, s, sel, g.thr);
    }
    return dev(e);
}

// Both forms are enqueued; each starts by reading the sampled zero counts and returns at once unless
// they select it, so exactly one of them computes dw.  No host synchronisation is involved.
st_status run_bww_auto(const st_conv_desc *d, const float *x, const float *dy, float *dw, void *ws,
                       size_t ws_bytes, void *stream)
{
    Dims o;
    st_status rc = validate(d, &o);
    if (rc != ST_OK) return rc;
    if ((rc = tensors_ok(x, dy, dw)) != ST_OK) return rc;
    if ((long long)d->K * d->S * d->R > 0x7fffffffLL) return ST_ERR_UNSUPPORTED;
    if (!ws_ok(ws, ws_bytes, workspace_bytes(*d, o, ST_PASS_BWW_AUTO, false))) return ST_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned *sel = static_cast<unsigned *>(ws);
    float *part = reinterpret_cast<float *>(static_cast<char *>(ws) + kCounterBytes);
    // Stride-2 3x3 layers: x has four times the elements of dy and each feeds 2.25 taps on average
    // (Sec. 3.3 of the paper), so the dy-testing form is the faster one whatever the two sparsities
    // (measured: 132 us with no zeros in dy against 157 us with 90 % zeros in x on 256->256 @28);
    // it is taken without sampling.
    if (d->stride_w == 2 && d->stride_h == 2 && st::bww_dy_fast_supported(*d))
        return dev(st::launch_bww_sparse_dy(*d, x, dy, dw, part, s));
    const size_t nx = (size_t)d->N * d->C * d->H * d->W, ny = (size_t)d->N * d->K * o.OH * o.OW;
    // the dense form takes part in the choice where tiled kernels exist for all three
    const bool tiled = st::bww_fast_supported(*d) && st::bww_dy_fast_supported(*d);
    const unsigned dense_thr = tiled ? st::bww_sparse_threshold(*d) : 0;
    if (dense_thr > 1000) return dev(st::launch_bww_dense(*d, x, dy, dw, part, s));    // never zero-skipping: unsampled
    if (st::launch_zero_sample(x, nx, dy, ny, sel, s, dense_thr) != hipSuccess) return ST_ERR_DEVICE;
    if (dense_thr != 0 && st::bww_auto_merged_supported(*d)) return dev(st::launch_bww_auto_merged(*d, x, dy, dw, part, s, sel));
    hipError_t e = st::bww_fast_supported(*d) ? st::launch_bww_sparse(*d, x, dy, dw, part, s, sel)
                                              : st::launch_generic_bww(*d, x, dy, dw, true, s, sel);
    if (e != hipSuccess) return ST_ERR_DEVICE;
    e = st::bww_dy_fast_supported(*d) ? st::launch_bww_sparse_dy(*d, x, dy, dw, part, s, sel)
                                      : st::launch_generic_bww_dy(*d, x, dy, dw, s, sel);
    if (e != hipSuccess || dense_thr == 0) return dev(e);
    return dev(st::launch_bww_dense(*d, x, dy, dw, part, s, sel));
}

// Device address of the built-in scratch array on the current device, looked up on the first call on
// that device and kept; nullptr (with *err set) if the runtime refuses.
float *static_scratch(hipError_t *err)
{
    static std::mutex lock;
    static float *ptr[st::kMaxDevices] = {};
    int devid = 0;
    *err = hipGetDevice(&devid);
    if (*err != hipSuccess) return nullptr;
    if (devid < 0 || devid >= st::kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
    std::lock_guard<std::mutex> hold(lock);
    if (!ptr[devid]) {
        void *p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (*err != hipSuccess || !p) { if (*err == hipSuccess) *err = hipErrorInvalidSymbol; return nullptr; }
        ptr[devid] = static_cast<float *>(p);
    }
    return ptr[devid];
}

}  // namespace

extern "C" {

st_status st_conv_fwd_static(const st_conv_desc *desc, const float *x, const float *w, float *y, void *hip_stream)
{
    Dims o;
    st_status rc = validate(desc, &o);
    if (rc != ST_OK) return rc;
    if ((rc = tensors_ok(x, w, y)) != ST_OK) return rc;
    const size_t need = workspace_bytes(*desc, o, ST_PASS_FWD, false);
    if (need > kStaticScratchBytes) return ST_ERR_WORKSPACE;
    if (need == 0) return run_fwd(desc, x, w, y, nullptr, 0, hip_stream, false);
    hipError_t e;
    float *ws = static_scratch(&e);
    if (!ws) return ST_ERR_DEVICE;
    return run_fwd(desc, x, w, y, ws, kStaticScratchBytes, hip_stream, false);
}

st_status st_conv_fwd(const st_conv_desc *desc, const float *x, const float *w, float *y, void *ws,
                      size_t ws_bytes, void *hip_stream)
{
    return run_fwd(desc, x, w, y, ws, ws_bytes, hip_stream, false);
}

st_status st_conv_fwd_dense(const st_conv_desc *desc, const float *x, const float *w, float *y,
                            void *ws, size_t ws_bytes, void *hip_stream)
{
    return run_fwd(desc, x, w, y, ws, ws_bytes, hip_stream, true);
}

st_status st_conv_bwi(const st_conv_desc *desc, const float *dy, const float *w, float *dx, void *ws,
                      size_t ws_bytes, void *hip_stream)
{
    return run_bwi(desc, dy, w, dx, ws, ws_bytes, hip_stream, false);
}

st_status st_conv_bwi_dense(const st_conv_desc *desc, const float *dy, const float *w, float *dx,
                            void *ws, size_t ws_bytes, void *hip_stream)
{
    return run_bwi(desc, dy, w, dx, ws, ws_bytes, hip_stream, true);
}

st_status st_conv_bww(const st_conv_desc *desc, const float *x, const float *dy, float *dw, void *ws,
                      size_t ws_bytes, void *hip_stream)
{
    return run_bww(desc, x, dy, dw, ws, ws_bytes, hip_stream, false);
}

st_status st_conv_bww_dy(const st_conv_desc *desc, const float *x, const float *dy, float *dw, void *ws,
                         size_t ws_bytes, void *hip_stream)
{
    return run_bww_dy(desc, x, dy, dw, ws, ws_bytes, hip_stream);
}

st_status st_conv_fwd_auto(const st_conv_desc *desc, const float *x, const float *w, float *y, void *ws,
                           size_t ws_bytes, void *hip_stream)
{
    return run_fwd_bwi_auto(desc, x, w, y, ws, ws_bytes, hip_stream, false);
}

st_status st_conv_bwi_auto(const st_conv_desc *desc, const float *dy, const float *w, float *dx, void *ws,
                           size_t ws_bytes, void *hip_stream)
{
    return run_fwd_bwi_auto(desc, dy, w, dx, ws, ws_bytes, hip_stream, true);
}

st_status st_conv_bww_auto(const st_conv_desc *desc, const float *x, const float *dy, float *dw, void *ws,
                           size_t ws_bytes, void *hip_stream)
{
    return run_bww_auto(desc, x, dy, dw, ws, ws_bytes, hip_stream);
}

st_status st_conv_bww_dense(const st_conv_desc *desc, const float *x, const float *dy, float *dw,
                            void *ws, size_t ws_bytes, void *hip_stream)
{
    return run_bww(desc, x, dy, dw, ws, ws_bytes, hip_stream, true);
}

size_t st_conv_workspace_bytes(const st_conv_desc *desc, int pass, int dense)
{
    Dims o;
    if (validate(desc, &o) != ST_OK) return 0;
    return workspace_bytes(*desc, o, pass, dense != 0);
}

int st_conv_sparse_threshold(const st_conv_desc *desc, int pass)
{
    Dims o;
    if (validate(desc, &o) != ST_OK) return -1;
    Geom g = fwd_geom(*desc, o);
    if (pass == ST_PASS_BWI || pass == ST_PASS_BWI_AUTO) {
        if (!bwi_as_fwd(*desc, o, &g)) return 0;
    } else if (pass != ST_PASS_FWD && pass != ST_PASS_FWD_AUTO) {
        return -1;
    }
    if (!st::fwd_sparse_supported(g) || !st::fwd_dense_supported(g)) return 0;
    return (int)st::fwd_sparse_threshold(g);
}

st_status st_conv_kernel_name(const st_conv_desc *desc, int pass, char *buf, size_t len)
{
    Dims o;
    st_status rc = validate(desc, &o);
    if (rc != ST_OK) return rc;
    if (!buf || len == 0) return ST_ERR_NULL;
    if (pass == ST_PASS_BWW) {
        if (!st::bww_fast_supported(*desc)) return ST_ERR_UNSUPPORTED;
        st::bww_sparse_kernel_name(*desc, buf, len);
        return ST_OK;
    }
    Geom g = fwd_geom(*desc, o);
    if (pass == ST_PASS_BWI || pass == ST_PASS_BWI_AUTO) {
        if (!bwi_as_fwd(*desc, o, &g)) return ST_ERR_UNSUPPORTED;
    } else if (pass != ST_PASS_FWD && pass != ST_PASS_FWD_AUTO) {
        return ST_ERR_UNSUPPORTED;
    }
    if (pass == ST_PASS_FWD_AUTO || pass == ST_PASS_BWI_AUTO) {
        // the single main kernel that holds both forms, where one exists for the geometry
        if (!st::fwd_auto_combined_supported(g)) return ST_ERR_UNSUPPORTED;
        st::fwd_auto_kernel_name(g, buf, len);
        return ST_OK;
    }
    if (!st::fwd_sparse_supported(g)) return ST_ERR_UNSUPPORTED;
    buf[0] = 0;
    g.describe = buf;
    g.describe_len = (int)(len > 0x7fffffff ? 0x7fffffff : len);
    return dev(st::launch_fwd_sparse(g, nullptr, nullptr, nullptr, nullptr));
}

const char *st_status_str(st_status status)
{
    switch (status) {
    case ST_OK: return "ok";
    case ST_ERR_NULL: return "a required pointer is NULL";
    case ST_ERR_BAD_SHAPE: return "bad shape: non-positive dimension, C or K not a multiple of 16, or empty output";
    case ST_ERR_UNSUPPORTED: return "shape not supported by any kernel";
    case ST_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case ST_ERR_DEVICE: return "HIP launch failed";
    case ST_ERR_ALIGNMENT: return "a tensor pointer is not 64-byte aligned";
    default: return "unknown status";
    }
}

const char *st_conv_version(void) { return "0.6"; }

}  // extern "C"
