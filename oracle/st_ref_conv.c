/*
 * st_ref_conv.c -- CPU oracle for the three convolution passes of CNN training.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * convolution passes compute.  It is used by the tests, by the smoke check and
 * by the "cpu_baseline" leg of the benchmark; the GPU library never links,
 * loads or calls it, and it shares no source with the GPU library.
 *
 * What is computed (SparseTrain, arXiv 1911.10175):
 *   FWD  Sec. 2.1, Eq. (1): the layer correlates K filters with the images.
 *   BWI  Sec. 2.1 (text after Eq. (2)): the gradient w.r.t. the layer input is
 *        the correlation of dL/dY with the transposed filters.
 *   BWW  Sec. 2.1 (same passage): the gradient w.r.t. the filters is the
 *        correlation of the input with dL/dY, S x R values per (c,k) pair.
 * The zero-skipping method of the paper (Algorithms 1 and 4) drops only
 * products whose tested factor compares equal to zero, so it reaches exactly
 * the dense result; the oracle proper is therefore the plain definition
 * ("gather" form, one output at a time).  The paper's input-stationary
 * forms with the zero test (Alg. 1, its BWI twin, Alg. 4: the tested operand is
 * visited element by element and a zero is dropped with all its products) are
 * also written out here, so that a test can check that they agree with the
 * definition and count what they skip.
 *
 * Symbols follow the paper's Table 1: N minibatch, C input channels, K output
 * channels, H x W input size, R filter WIDTH (pairs with W, iterator u),
 * S filter HEIGHT (pairs with H, iterator v), O horizontal stride (stride_w),
 * P vertical stride (stride_h).  The paper never mentions padding; here it is
 * explicit and symmetric (pad_w left and right, pad_h top and bottom), and a
 * read outside the image yields 0 / an update outside the output is dropped.
 *
 * Plain row-major layouts (NOT the blocked layout of the GPU library):
 *   x, dx : [N][C][H][W]        y, dy : [N][K][OH][OW]
 *   w, dw : [K][C][S][R]        (height index v before width index u)
 *   OH = (H + 2 pad_h - S) / P + 1,  OW = (W + 2 pad_w - R) / O + 1.
 *
 * Arithmetic: inputs are fp32; every product is formed in fp64 (exact, since
 * 24 + 24 <= 53 significand bits) and summed in fp64.  Each gather routine
 * also returns abs = sum of |product| per output, the scale against which the
 * GPU result's error is measured.
 *
 * Pins (tests/test_oracle_*.py): brute-force loops over explicitly padded
 * arrays on tiny non-square shapes, a hand-worked instance of Eq. (1), the
 * tap-count closed form for all-ones tensors, the identity filter, the 1x1
 * case against a matrix product, a library fp64 convolution, the adjoint
 * identities <FWD(x,w),dy> = <x,BWI(dy,w)> = <w,BWW(x,dy)>, the rotated /
 * transposed-filter identity for stride-1 BWI, and scatter == gather.
 *
 * Every function returns 0 on success and a negative number on bad arguments.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* dims[11] = N, C, K, H, W, R, S, stride_w (O), stride_h (P), pad_w, pad_h */
typedef struct {
    int N, C, K, H, W, R, S, O, P, pad_w, pad_h, OH, OW;
} ref_geom;

static int ref_geom_init(ref_geom *g, const int32_t *d)
{
    if (!d) return -1;
    g->N = d[0]; g->C = d[1]; g->K = d[2]; g->H = d[3]; g->W = d[4];
    g->R = d[5]; g->S = d[6]; g->O = d[7]; g->P = d[8];
    g->pad_w = d[9]; g->pad_h = d[10];
    if (g->N <= 0 || g->C <= 0 || g->K <= 0 || g->H <= 0 || g->W <= 0) return -2;
    if (g->R <= 0 || g->S <= 0 || g->O <= 0 || g->P <= 0) return -2;
    if (g->pad_w < 0 || g->pad_h < 0) return -2;
    if (g->H + 2 * g->pad_h < g->S || g->W + 2 * g->pad_w < g->R) return -3;
    g->OH = (g->H + 2 * g->pad_h - g->S) / g->P + 1;
    g->OW = (g->W + 2 * g->pad_w - g->R) / g->O + 1;
    return 0;
}

int st_ref_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int st_ref_out_dims(const int32_t *dims, int32_t *oh, int32_t *ow)
{
    ref_geom g;
    int rc = ref_geom_init(&g, dims);
    if (rc) return rc;
    if (oh) *oh = g.OH;
    if (ow) *ow = g.OW;
    return 0;
}

#define X_AT(g, n, c, h, w) ((((size_t)(n) * (g).C + (c)) * (g).H + (h)) * (g).W + (w))
#define Y_AT(g, n, k, oh, ow) ((((size_t)(n) * (g).K + (k)) * (g).OH + (oh)) * (g).OW + (ow))
#define W_AT(g, k, c, v, u) ((((size_t)(k) * (g).C + (c)) * (g).S + (v)) * (g).R + (u))

/* ---- FWD, Eq. (1): one output element ---------------------------------- */
static void fwd_one(const ref_geom *g, const float *x, const float *w,
                    int n, int k, int oh, int ow, double *sum, double *asum)
{
    double s = 0.0, a = 0.0;
    for (int c = 0; c < g->C; ++c)
        for (int v = 0; v < g->S; ++v) {
            int ih = oh * g->P - g->pad_h + v;
            if (ih < 0 || ih >= g->H) continue;
            for (int u = 0; u < g->R; ++u) {
                int iw = ow * g->O - g->pad_w + u;
                if (iw < 0 || iw >= g->W) continue;
                double t = (double)x[X_AT(*g, n, c, ih, iw)] * (double)w[W_AT(*g, k, c, v, u)];
                s += t;
                a += fabs(t);
            }
        }
    *sum = s;
    *asum = a;
}

/* ---- BWI: one input-gradient element ----------------------------------- */
/* dx[n,c,ih,iw] collects dy[n,k,oh,ow] * w[k,c,v,u] over every (k,v,u,oh,ow)
 * for which the forward pass read x[n,c,ih,iw] through tap (v,u), i.e.
 * oh*P - pad_h + v == ih and ow*O - pad_w + u == iw. */
static void bwi_one(const ref_geom *g, const float *dy, const float *w,
                    int n, int c, int ih, int iw, double *sum, double *asum)
{
    double s = 0.0, a = 0.0;
    for (int k = 0; k < g->K; ++k)
        for (int v = 0; v < g->S; ++v) {
            int th = ih + g->pad_h - v;
            if (th < 0 || th % g->P) continue;
            int oh = th / g->P;
            if (oh >= g->OH) continue;
            for (int u = 0; u < g->R; ++u) {
                int tw = iw + g->pad_w - u;
                if (tw < 0 || tw % g->O) continue;
                int ow = tw / g->O;
                if (ow >= g->OW) continue;
                double t = (double)dy[Y_AT(*g, n, k, oh, ow)] * (double)w[W_AT(*g, k, c, v, u)];
                s += t;
                a += fabs(t);
            }
        }
    *sum = s;
    *asum = a;
}

/* ---- BWW: one filter-gradient element ---------------------------------- */
static void bww_one(const ref_geom *g, const float *x, const float *dy,
                    int k, int c, int v, int u, double *sum, double *asum)
{
    double s = 0.0, a = 0.0;
    for (int n = 0; n < g->N; ++n)
        for (int oh = 0; oh < g->OH; ++oh) {
            int ih = oh * g->P - g->pad_h + v;
            if (ih < 0 || ih >= g->H) continue;
            for (int ow = 0; ow < g->OW; ++ow) {
                int iw = ow * g->O - g->pad_w + u;
                if (iw < 0 || iw >= g->W) continue;
                double t = (double)x[X_AT(*g, n, c, ih, iw)] * (double)dy[Y_AT(*g, n, k, oh, ow)];
                s += t;
                a += fabs(t);
            }
        }
    *sum = s;
    *asum = a;
}

/* ======================= full-tensor gather forms ======================== */

int st_ref_conv_fwd(const int32_t *dims, const float *x, const float *w,
                    double *y, double *y_abs)
{
    ref_geom g;
    int rc = ref_geom_init(&g, dims);
    if (rc) return rc;
    if (!x || !w || !y) return -1;
    long long total = (long long)g.N * g.K * g.OH;
#pragma omp parallel for schedule(static)
    for (long long t = 0; t < total; ++t) {
        int oh = (int)(t % g.OH);
        int k = (int)((t / g.OH) % g.K);
        int n = (int)(t / ((long long)g.OH * g.K));
        for (int ow = 0; ow < g.OW; ++ow) {
            double s, a;
            fwd_one(&g, x, w, n, k, oh, ow, &s, &a);
            size_t o = Y_AT(g, n, k, oh, ow);
            y[o] = s;
            if (y_abs) y_abs[o] = a;
        }
    }
    return 0;
}

int st_ref_conv_bwi(const int32_t *dims, const float *dy, const float *w,
                    double *dx, double *dx_abs)
{
    ref_geom g;
    int rc = ref_geom_init(&g, dims);
    if (rc) return rc;
    if (!dy || !w || !dx) return -1;
    long long total = (long long)g.N * g.C * g.H;
#pragma omp parallel for schedule(static)
    for (long long t = 0; t < total; ++t) {
        int ih = (int)(t % g.H);
        int c = (int)((t / g.H) % g.C);
        int n = (int)(t / ((long long)g.H * g.C));
        for (int iw = 0; iw < g.W; ++iw) {
            double s, a;
            bwi_one(&g, dy, w, n, c, ih, iw, &s, &a);
            size_t o = X_AT(g, n, c, ih, iw);
            dx[o] = s;
            if (dx_abs) dx_abs[o] = a;
        }
    }
    return 0;
}

int st_ref_conv_bww(const int32_t *dims, const float *x, const float *dy,
                    double *dw, double *dw_abs)
{
    ref_geom g;
    int rc = ref_geom_init(&g, dims);
    if (rc) return rc;
    if (!x || !dy || !dw) return -1;
    long long total = (long long)g.K * g.C;
#pragma omp parallel for schedule(dynamic, 1)
    for (long long t = 0; t < total; ++t) {
        int c = (int)(t % g.C);
        int k = (int)(t / g.C);
        for (int v = 0; v < g.S; ++v)
            for (int u = 0; u < g.R; ++u) {
                double s, a;
                bww_one(&g, x, dy, k, c, v, u, &s, &a);
                size_t o = W_AT(g, k, c, v, u);
                dw[o] = s;
                if (dw_abs) dw_abs[o] = a;
            }
    }
    return 0;
}

/* ================== sampled gather forms (large tensors) ================= */
/* coords holds 4 int32 per sample.  FWD: (n,k,oh,ow); BWI: (n,c,ih,iw);
 * BWW: (k,c,v,u).  out/out_abs hold one double per sample. */

int st_ref_conv_fwd_at(const int32_t *dims, const float *x, const float *w,
                       int64_t n_samples, const int32_t *coords,
                       double *out, double *out_abs)
{
    ref_geom g;
    int rc = ref_geom_init(&g, dims);
    if (rc) return rc;
    if (!x || !w || !coords || !out) return -1;
    for (int64_t i = 0; i < n_samples; ++i) {
        const int32_t *q = coords + 4 * i;
        if (q[0] < 0 || q[0] >= g.N || q[1] < 0 || q[1] >= g.K ||
            q[2] < 0 || q[2] >= g.OH || q[3] < 0 || q[3] >= g.OW) return -4;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_samples; ++i) {
        const int32_t *q = coords + 4 * i;
        double s, a;
        fwd_one(&g, x, w, q[0], q[1], q[2], q[3], &s, &a);
        out[i] = s;
        if (out_abs) out_abs[i] = a;
    }
    return 0;
}

int st_ref_conv_bwi_at(const int32_t *dims, const float *dy, const float *w,
                       int64_t n_samples, const int32_t *coords,
                       double *out, double *out_abs)
{
    ref_geom g;
    int rc = ref_geom_init(&g, dims);
    if (rc) return rc;
    if (!dy || !w || !coords || !out) return -1;
    for (int64_t i = 0; i < n_samples; ++i) {
        const int32_t *q = coords + 4 * i;
        if (q[0] < 0 || q[0] >= g.N || q[1] < 0 || q[1] >= g.C ||
            q[2] < 0 || q[2] >= g.H || q[3] < 0 || q[3] >= g.W) return -4;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_samples; ++i) {
        const int32_t *q = coords + 4 * i;
        double s, a;
        bwi_one(&g, dy, w, q[0], q[1], q[2], q[3], &s, &a);
        out[i] = s;
        if (out_abs) out_abs[i] = a;
    }
    return 0;
}

int st_ref_conv_bww_at(const int32_t *dims, const float *x, const float *dy,
                       int64_t n_samples, const int32_t *coords,
                       double *out, double *out_abs)
{
    ref_geom g;
    int rc = ref_geom_init(&g, dims);
    if (rc) return rc;
    if (!x || !dy || !coords || !out) return -1;
    for (int64_t i = 0; i < n_samples; ++i) {
        const int32_t *q = coords + 4 * i;
        if (q[0] < 0 || q[0] >= g.K || q[1] < 0 || q[1] >= g.C ||
            q[2] < 0 || q[2] >= g.S || q[3] < 0 || q[3] >= g.R) return -4;
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_samples; ++i) {
        const int32_t *q = coords + 4 * i;
        double s, a;
        bww_one(&g, x, dy, q[0], q[1], q[2], q[3], &s, &a);
        out[i] = s;
        if (out_abs) out_abs[i] = a;
    }
    return 0;
}

/* ============ the zero-skipping forms (tested operand stationary) ========= */
/* Sec. 3.1 (Alg. 1) and Sec. 3.4 (Alg. 4) visit the tested operand element by
 * element, drop an element that compares equal to zero together with all of
 * its products, and add the products of every other element to the outputs
 * they belong to.  The test is the IEEE comparison "value != 0": +0 and -0
 * are dropped, denormals are not (Alg. 3 builds its mask with a vector compare
 * against 0).  These routines are organised around the list of (tap, partner
 * pixel) pairs of one tested pixel, which is all the geometry there is; the
 * channel loop of the untested side is innermost.  Serial on purpose: updates
 * to one output come from many tested elements.  *n_skipped (optional)
 * receives the number of tested elements that were dropped. */

typedef struct { int v, u, ph, pw; } ref_link;     /* tap (v,u) and the partner pixel (ph,pw) */

/* Pairs of an INPUT pixel (ih,iw): output pixel (oh,ow) reads it through tap
 * (v,u) iff oh*P - pad_h + v == ih and ow*O - pad_w + u == iw.  With unit
 * strides and no padding this is the paper's Y[x-u, y-v].  Returns the count
 * (at most S*R). */
static int links_of_input_pixel(const ref_geom *g, int ih, int iw, ref_link *l)
{
    int n = 0;
    for (int v = 0; v < g->S; ++v) {
        int th = ih + g->pad_h - v;
        if (th < 0 || th % g->P || th / g->P >= g->OH) continue;
        for (int u = 0; u < g->R; ++u) {
            int tw = iw + g->pad_w - u;
            if (tw < 0 || tw % g->O || tw / g->O >= g->OW) continue;
            l[n].v = v; l[n].u = u; l[n].ph = th / g->P; l[n].pw = tw / g->O;
            ++n;
        }
    }
    return n;
}

/* Pairs of an OUTPUT pixel (oh,ow): the input pixels its taps read. */
static int links_of_output_pixel(const ref_geom *g, int oh, int ow, ref_link *l)
{
    int n = 0;
    for (int v = 0; v < g->S; ++v) {
        int ih = oh * g->P - g->pad_h + v;
        if (ih < 0 || ih >= g->H) continue;
        for (int u = 0; u < g->R; ++u) {
            int iw = ow * g->O - g->pad_w + u;
            if (iw < 0 || iw >= g->W) continue;
            l[n].v = v; l[n].u = u; l[n].ph = ih; l[n].pw = iw;
            ++n;
        }
    }
    return n;
}

enum { REF_MAX_TAPS = 1024 };

/* FWD with the zero test on x (Sec. 3.1, Alg. 1). */
int st_ref_conv_fwd_scatter(const int32_t *dims, const float *x, const float *w,
                            double *y, int64_t *n_skipped)
{
    ref_geom g;
    int rc = ref_geom_init(&g, dims);
    if (rc) return rc;
    if (!x || !w || !y) return -1;
    if ((int64_t)g.S * g.R > REF_MAX_TAPS) return -5;
    ref_link l[REF_MAX_TAPS];
    memset(y, 0, (size_t)g.N * g.K * g.OH * g.OW * sizeof(double));
    int64_t skipped = 0;
    const int64_t total = (int64_t)g.N * g.C * g.H * g.W;
    for (int64_t e = 0; e < total; ++e) {           /* e = flat index into x[N][C][H][W] */
        const float d = x[e];
        if (!(d != 0.0f)) { ++skipped; continue; }
        const int iw = (int)(e % g.W), ih = (int)(e / g.W % g.H);
        const int c = (int)(e / ((int64_t)g.W * g.H) % g.C), n = (int)(e / ((int64_t)g.W * g.H * g.C));
        const int nl = links_of_input_pixel(&g, ih, iw, l);
        for (int i = 0; i < nl; ++i)
            for (int k = 0; k < g.K; ++k)
                y[Y_AT(g, n, k, l[i].ph, l[i].pw)] += (double)d * (double)w[W_AT(g, k, c, l[i].v, l[i].u)];
    }
    if (n_skipped) *n_skipped = skipped;
    return 0;
}

/* BWI with the zero test on dy (Sec. 3.1 treats BWI like FWD): each non-zero
 * dy element is spread over the input pixels it was computed from, the filter
 * being indexed by the input channel. */
int st_ref_conv_bwi_scatter(const int32_t *dims, const float *dy, const float *w,
                            double *dx, int64_t *n_skipped)
{
    ref_geom g;
    int rc = ref_geom_init(&g, dims);
    if (rc) return rc;
    if (!dy || !w || !dx) return -1;
    if ((int64_t)g.S * g.R > REF_MAX_TAPS) return -5;
    ref_link l[REF_MAX_TAPS];
    memset(dx, 0, (size_t)g.N * g.C * g.H * g.W * sizeof(double));
    int64_t skipped = 0;
    const int64_t total = (int64_t)g.N * g.K * g.OH * g.OW;
    for (int64_t e = 0; e < total; ++e) {           /* e = flat index into dy[N][K][OH][OW] */
        const float d = dy[e];
        if (!(d != 0.0f)) { ++skipped; continue; }
        const int ow = (int)(e % g.OW), oh = (int)(e / g.OW % g.OH);
        const int k = (int)(e / ((int64_t)g.OW * g.OH) % g.K), n = (int)(e / ((int64_t)g.OW * g.OH * g.K));
        const int nl = links_of_output_pixel(&g, oh, ow, l);
        for (int i = 0; i < nl; ++i)
            for (int c = 0; c < g.C; ++c)
                dx[X_AT(g, n, c, l[i].ph, l[i].pw)] += (double)d * (double)w[W_AT(g, k, c, l[i].v, l[i].u)];
    }
    if (n_skipped) *n_skipped = skipped;
    return 0;
}

/* BWW with the zero test on x (Sec. 3.4, Alg. 4; test_dy = 0) or on dy
 * (test_dy = 1: the variant Sec. 3.4 mentions for layers whose dy is the
 * sparser operand). */
int st_ref_conv_bww_scatter(const int32_t *dims, const float *x, const float *dy,
                            int test_dy, double *dw, int64_t *n_skipped)
{
    ref_geom g;
    int rc = ref_geom_init(&g, dims);
    if (rc) return rc;
    if (!x || !dy || !dw) return -1;
    if ((int64_t)g.S * g.R > REF_MAX_TAPS) return -5;
    ref_link l[REF_MAX_TAPS];
    memset(dw, 0, (size_t)g.K * g.C * g.S * g.R * sizeof(double));
    int64_t skipped = 0;
    if (!test_dy) {
        const int64_t total = (int64_t)g.N * g.C * g.H * g.W;
        for (int64_t e = 0; e < total; ++e) {
            const float d = x[e];
            if (!(d != 0.0f)) { ++skipped; continue; }
            const int iw = (int)(e % g.W), ih = (int)(e / g.W % g.H);
            const int c = (int)(e / ((int64_t)g.W * g.H) % g.C), n = (int)(e / ((int64_t)g.W * g.H * g.C));
            const int nl = links_of_input_pixel(&g, ih, iw, l);
            for (int i = 0; i < nl; ++i)
                for (int k = 0; k < g.K; ++k)
                    dw[W_AT(g, k, c, l[i].v, l[i].u)] += (double)d * (double)dy[Y_AT(g, n, k, l[i].ph, l[i].pw)];
        }
    } else {
        const int64_t total = (int64_t)g.N * g.K * g.OH * g.OW;
        for (int64_t e = 0; e < total; ++e) {
            const float d = dy[e];
            if (!(d != 0.0f)) { ++skipped; continue; }
            const int ow = (int)(e % g.OW), oh = (int)(e / g.OW % g.OH);
            const int k = (int)(e / ((int64_t)g.OW * g.OH) % g.K), n = (int)(e / ((int64_t)g.OW * g.OH * g.K));
            const int nl = links_of_output_pixel(&g, oh, ow, l);
            for (int i = 0; i < nl; ++i)
                for (int c = 0; c < g.C; ++c)
                    dw[W_AT(g, k, c, l[i].v, l[i].u)] += (double)x[X_AT(g, n, c, l[i].ph, l[i].pw)] * (double)d;
        }
    }
    if (n_skipped) *n_skipped = skipped;
    return 0;
}
