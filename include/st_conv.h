/*
 * st_conv.h -- C ABI of the MI355X (gfx950) zero-skipping convolution library.
 *
 * The library computes the three direct-convolution passes of CNN training
 * described in SparseTrain (arXiv 1911.10175): forward (FWD), backward by
 * input (BWI) and backward by weights (BWW).  The st_conv_{fwd,bwi,bww} entry
 * points test one operand for zeros on the fly and skip every multiply-add
 * that zero would feed (Sec. 3 of the paper); the st_conv_*_dense entry points
 * compute the same tensors with no test and no skipping and serve as the
 * dense control.  All tensors stay in a dense, fixed, blocked fp32 layout
 * (Sec. 3 opening: the data representation is dense; Sec. 3.2.5: the lowest
 * dimension is a channel tile).
 *
 * Symbols (Table 1 of the paper): N minibatch, C input channels, K output
 * channels, H x W input height x width, R filter WIDTH (pairs with W),
 * S filter HEIGHT (pairs with H), O = stride_w, P = stride_h.  The paper leaves
 * padding implicit; here it is explicit and symmetric per axis.
 *   OH = (H + 2*pad_h - S) / stride_h + 1,  OW = (W + 2*pad_w - R) / stride_w + 1.
 *
 * Layouts (fp32, channel block B = 16; every pointer is a DEVICE pointer,
 * 64-byte aligned, row-major in the listed order):
 *   activations and their gradients   x, dx : [N][C/16][H ][W ][16 c]
 *                                      y, dy : [N][K/16][OH][OW][16 k]
 *   filters and their gradients        w, dw : [K/16][C/16][S][R][16 c][16 k]
 * (Sec. 3.2.5 fixes the lowest dimensions: channel tile for activations;
 *  k vector, then c tile, then the filter-width index for filters.)
 *
 * Ownership and execution: the caller owns every buffer, the workspace
 * included.  The library never allocates, frees or synchronises; each call
 * enqueues kernels on the given HIP stream (a hipStream_t passed as void*,
 * NULL = the default stream) and returns.  Outputs are overwritten (beta = 0).
 * Inputs are read-only.  Buffers must not overlap.
 *
 * Errors: every entry point returns a status and never aborts, throws or
 * prints.  Arguments are checked on the host before anything is enqueued:
 * descriptor, NULL and misaligned tensor pointers (ST_ERR_ALIGNMENT: the
 * kernels use 16-byte vector accesses, which would fault), workspace.  With
 * every status except ST_OK and ST_ERR_DEVICE nothing has been enqueued.
 * ST_ERR_DEVICE means the HIP runtime refused one of the call's launches; a
 * pass is up to seven launches (filter copy, sampling, main kernels, final
 * sums), so earlier ones may already be in the stream: the contents of the
 * output and of the workspace are then undefined.
 *
 * Limits (ST_ERR_UNSUPPORTED beyond them): H*W and OH*OW at most 2^27 - 1
 * pixels, C*S*R (and K*S*R for the dy-testing BWW forms) at most 2^31 - 1,
 * N at most 65535.
 *
 * The library reads no environment variables; kernel shapes and reduction
 * splits depend on the descriptor alone.
 *
 * Numerics: products and sums are fp32; the summation order is unspecified
 * but fixed for a given shape (results are run-to-run deterministic; no
 * floating-point atomics).  A skipped term is one whose tested factor compares
 * equal to zero (IEEE: +0 and -0; denormals are NOT flushed before the test).
 * With finite inputs the sparse and dense entry points agree to rounding; with
 * non-finite inputs they may differ (0 * Inf is skipped, not NaN).
 */
#ifndef ST_CONV_H
#define ST_CONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ST_OK = 0,
    ST_ERR_NULL = 1,        /* a required pointer is NULL */
    ST_ERR_BAD_SHAPE = 2,   /* non-positive dimension, C or K not a multiple of 16, empty output */
    ST_ERR_UNSUPPORTED = 3, /* a well-formed shape that no kernel covers */
    ST_ERR_WORKSPACE = 4,   /* workspace missing, misaligned or smaller than st_conv_workspace_bytes */
    ST_ERR_DEVICE = 5,      /* the HIP runtime refused a launch */
    ST_ERR_ALIGNMENT = 6    /* a tensor pointer is not 64-byte aligned */
} st_status;

/* Convolution geometry, Table 1 of the paper plus explicit padding. */
typedef struct {
    int32_t N, C, K;
    int32_t H, W;               /* input height, width */
    int32_t R, S;               /* filter width (u), filter height (v) */
    int32_t stride_w, stride_h; /* O, P */
    int32_t pad_w, pad_h;       /* zeros added on each side of W / of H */
} st_conv_desc;

enum {
    ST_PASS_FWD = 0, ST_PASS_BWI = 1, ST_PASS_BWW = 2, ST_PASS_BWW_DY = 3, ST_PASS_BWW_AUTO = 4,
    ST_PASS_FWD_AUTO = 5, ST_PASS_BWI_AUTO = 6
};

/*
 * FWD, Eq. (1) of Sec. 2.1 (correlation, filter not flipped, no bias):
 *   y[n,k,oh,ow] = sum_{c,v,u} x[n,c,oh*P-pad_h+v, ow*O-pad_w+u] * w[k,c,v,u]
 * with reads outside the image equal to 0.  st_conv_fwd skips all products of
 * an x element that is zero (Sec. 3.1-3.2, Alg. 1-3).
 *   x  in   [N][C/16][H][W][16]           w  in  [K/16][C/16][S][R][16][16]
 *   y  out  [N][K/16][OH][OW][16]
 *   ws / ws_bytes: workspace of at least st_conv_workspace_bytes(desc, ST_PASS_FWD, dense)
 *                  bytes (may be NULL when that is 0).  The tiled kernels read the filters from a
 *                  copy in their own order which they write there first, on every call.
 */
st_status st_conv_fwd(const st_conv_desc *desc, const float *x, const float *w, float *y,
                      void *ws, size_t ws_bytes, void *hip_stream);
st_status st_conv_fwd_dense(const st_conv_desc *desc, const float *x, const float *w, float *y,
                            void *ws, size_t ws_bytes, void *hip_stream);

/*
 * BWI, Sec. 2.1 (passage after Eq. (2)) and Sec. 3.3: the gradient of the loss
 * w.r.t. the layer input is the correlation of dy with the transposed filters:
 *   dx[n,c,ih,iw] = sum_{k,v,u} dy[n,k,oh,ow] * w[k,c,v,u]
 *   over the (oh,ow) with oh*P-pad_h+v = ih and ow*O-pad_w+u = iw.
 * st_conv_bwi skips all products of a dy element that is zero.
 *   dy in   [N][K/16][OH][OW][16]         w  in  [K/16][C/16][S][R][16][16]
 *   dx out  [N][C/16][H][W][16]
 */
st_status st_conv_bwi(const st_conv_desc *desc, const float *dy, const float *w, float *dx,
                      void *ws, size_t ws_bytes, void *hip_stream);
st_status st_conv_bwi_dense(const st_conv_desc *desc, const float *dy, const float *w, float *dx,
                            void *ws, size_t ws_bytes, void *hip_stream);

/*
 * BWW, Sec. 2.1 (same passage) and Sec. 3.4 (Alg. 4-5): the gradient w.r.t.
 * the filters is the correlation of the input with dy:
 *   dw[k,c,v,u] = sum_{n,oh,ow} x[n,c,oh*P-pad_h+v, ow*O-pad_w+u] * dy[n,k,oh,ow].
 * st_conv_bww skips all products of an x element that is zero (the operand
 * Alg. 4 tests).  Partial sums over parts of the minibatch are kept in the
 * workspace and added by a second kernel in a fixed order (Sec. 3.4, last
 * paragraphs: partial results are accumulated at the end of a sweep).
 *   x  in   [N][C/16][H][W][16]           dy in  [N][K/16][OH][OW][16]
 *   dw out  [K/16][C/16][S][R][16][16]
 */
st_status st_conv_bww(const st_conv_desc *desc, const float *x, const float *dy, float *dw,
                      void *ws, size_t ws_bytes, void *hip_stream);
st_status st_conv_bww_dense(const st_conv_desc *desc, const float *x, const float *dy, float *dw,
                            void *ws, size_t ws_bytes, void *hip_stream);

/*
 * BWW with the zero test on dy instead of x: Sec. 3.4 notes that Alg. 4 is easily changed to check
 * dy when the layer's output gradient is the sparser operand, and Sec. 5.3 chooses per layer the
 * operand with the higher average sparsity.  Same tensors, same result as st_conv_bww; all products
 * of a dy element that is zero are skipped.  The choice is the caller's (it knows the layer's
 * statistics); workspace size: st_conv_workspace_bytes(desc, ST_PASS_BWW_DY, 0).
 */
st_status st_conv_bww_dy(const st_conv_desc *desc, const float *x, const float *dy, float *dw,
                         void *ws, size_t ws_bytes, void *hip_stream);

/*
 * BWW that picks the tested operand itself, per call: Sec. 5.3 tests the operand with the higher
 * average sparsity, and Sec. 5.4 names the fixed choice a limitation.  A first kernel counts the
 * zeros in a sample of x and of dy (at most 64 evenly spaced blocks of 1024 elements each); then
 * the forms above are enqueued, and those the counts do not select return at once: x is tested
 * unless the zero fraction of dy is larger by more than 3 percentage points (at equal fractions
 * the x-testing form is the faster one).  Same tensors, same result, no host
 * synchronisation; the cost is the sampling pass (at most 256 KB of x and of dy are read once more)
 * and the empty launches.  Where tiled kernels exist, the dense form (st_conv_bww_dense) is the
 * third candidate: it runs when even the sparser operand has fewer zeros than the measured
 * break-even, 25 % for 3x3 layers (Sec. 5.3 combines the kernels with dense ones layer by layer).
 * Two kinds of layer are decided without sampling: 1x1 layers, where a zero saves too few
 * multiply-adds to beat the matrix cores at any zero fraction measured (up to 95 %), go straight to the dense form;
 * stride-2 3x3 layers always test dy (x has four times the elements and each feeds fewer taps,
 * Sec. 3.3, so that form is the faster one at any sparsity).
 * Workspace: st_conv_workspace_bytes(desc, ST_PASS_BWW_AUTO, 0).
 */
st_status st_conv_bww_auto(const st_conv_desc *desc, const float *x, const float *dy, float *dw,
                           void *ws, size_t ws_bytes, void *hip_stream);

/*
 * FWD and BWI with the choice between the zero-skipping and the dense form made per call on the
 * device.  Sec. 5.3 of the paper combines its kernels with the dense ones layer by layer, from
 * profiled sparsity; here a first kernel counts the zeros in a sample of the tested operand (x for
 * FWD, dy for BWI; at most 64 evenly spaced blocks of 1024 elements) in the same launch that
 * writes both forms' filter copies, then both forms are enqueued and the one the count does not
 * select returns at once.  The zero-skipping form runs when the sampled zero fraction reaches the
 * break-even point measured for the geometry: 25 % for 3x3 layers with K a multiple of 128, 40 %
 * for narrower ones, 80 % / 45 % for FWD / BWI of stride-2 3x3 layers, never for 1x1 layers
 * (measured up to 95 % zeros), always for geometries only the generic kernels cover.  Where the answer is "always" or "never" the call
 * goes straight to that form, without sampling.  On unit-stride 3x3 layers of the usual sizes one
 * main kernel holds both forms and runs the selected one, so the sampled path has as many launches
 * as the direct call (st_conv_kernel_name tells); elsewhere it costs one launch more; a caller that tracks sparsity itself can compare it with st_conv_sparse_threshold
 * and call the form directly.  Same tensors and layouts as st_conv_fwd / st_conv_bwi, same result
 * to rounding, no host synchronisation.
 * Workspace: st_conv_workspace_bytes(desc, ST_PASS_FWD_AUTO or ST_PASS_BWI_AUTO, 0).
 */
st_status st_conv_fwd_auto(const st_conv_desc *desc, const float *x, const float *w, float *y,
                           void *ws, size_t ws_bytes, void *hip_stream);
st_status st_conv_bwi_auto(const st_conv_desc *desc, const float *dy, const float *w, float *dx,
                           void *ws, size_t ws_bytes, void *hip_stream);

/*
 * st_conv_fwd for callers that cannot allocate device memory or carry a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same tensors, same kernels
 * and bit-identical results as st_conv_fwd; the filter copy that st_conv_fwd writes into the caller's
 * workspace goes into a 16 MiB array built into the library's device image instead (one copy per GPU
 * the library runs on, held until the process ends).  The call allocates and frees nothing and does
 * not synchronise.  Geometries whose filter copy st_conv_workspace_bytes(desc, ST_PASS_FWD, 0)
 * exceeds 16 MiB (16777216 bytes) are refused with ST_ERR_WORKSPACE before anything is enqueued.
 * The first call on a device looks up the array's device address (ST_ERR_DEVICE if the runtime
 * refuses); make that call outside a graph capture.  All calls on one GPU share the one array, which
 * keeps the last call's filter copy: nothing in it has to start at zero (every element a launch
 * reads is written by the same call first), but two calls in flight at the same time on one GPU
 * - on different streams or from different threads - race on it and must be serialised by the caller.
 */
st_status st_conv_fwd_static(const st_conv_desc *desc, const float *x, const float *w, float *y,
                             void *hip_stream);

/*
 * Bytes of device workspace the given pass needs for this geometry
 * (pass = ST_PASS_*, dense = 0 for st_conv_<pass>, 1 for st_conv_<pass>_dense; ST_PASS_BWW_DY with
 * dense = 0 is st_conv_bww_dy, ST_PASS_*_AUTO with dense = 0 are the st_conv_*_auto entry points).
 * Returns 0 when none is needed or when desc is invalid (the pass itself then
 * reports the error).  The workspace must be 256-byte aligned.  Its contents
 * need not be initialised and are undefined afterwards; two calls that are in
 * flight at the same time must not share one.
 */
size_t st_conv_workspace_bytes(const st_conv_desc *desc, int pass, int dense);

/*
 * The zero fraction of the tested operand, in per mille, from which st_conv_fwd_auto (pass =
 * ST_PASS_FWD) or st_conv_bwi_auto (pass = ST_PASS_BWI) runs the zero-skipping form for this
 * geometry: 0 = always, 1001 = never; -1 for an invalid descriptor or another pass.  Host-side,
 * no GPU work.
 */
int st_conv_sparse_threshold(const st_conv_desc *desc, int pass);

/*
 * Name of the main kernel st_conv_fwd (pass = ST_PASS_FWD), st_conv_bwi (ST_PASS_BWI) or st_conv_bww
 * (ST_PASS_BWW) launches for this geometry, with its template arguments, as a profiler prints it (e.g.
 * "fwd_sparse_kernel<3, 3, 4, 8, 2, 4, 4, 1, 1, 0>": filter width, height, tile height, width, channels per
 * lane, wavefronts per SIMD aimed at, wavefronts sharing a tile, output stride, input spacing, input offset;
 * "bww_sparse_kernel<3, 3, 7, 8, 0>": filter width, height, tile height, width, stride mode).
 * With pass = ST_PASS_FWD_AUTO or ST_PASS_BWI_AUTO: the single main kernel of st_conv_fwd_auto /
 * st_conv_bwi_auto that holds both forms ("fwd_auto_kernel<4, 8, 2, 4, 4, 8>": tile height, width,
 * channels per lane and wavefronts per tile of the zero-skipping form, column blocks and tile width of
 * the dense one), ST_ERR_UNSUPPORTED where the two forms are launched separately.  For matching
 * profiler output and timings to calls; host side only, launches nothing.  buf receives at most len
 * bytes including the terminating NUL.  ST_ERR_UNSUPPORTED for other passes and for geometries the
 * generic kernels serve.
 */
st_status st_conv_kernel_name(const st_conv_desc *desc, int pass, char *buf, size_t len);

/*
 * Measurement aid, not part of the convolution path: runs a bare instruction stream that gives the issue
 * rate of the vector pipe for the operand patterns of the zero-skipping kernels (Sec. 3.1's broadcast
 * multiply-add, here v_fmac_f32 with the tested value as one source) or of the matrix pipe.
 *   pattern 0: 63 independent v_fmac_f32 per iteration, tested-value register changing every instruction
 *   pattern 1: the same with one tested-value register as FIRST source for nine instructions in a row
 *   pattern 2: the same with it as SECOND source
 *   pattern 3: 4 independent v_mfma_f32_32x32x2_f32 per iteration
 *   pattern 4: 63 v_fmac_f32 whose accumulator and two factors all sit in even-numbered registers
 *   pattern 5: the same accumulators and first factors with the second factor in odd-numbered registers
 * workgroups of 256 threads (4 wavefronts, one per SIMD), iters iterations each; out (device) receives one
 * float per thread, workgroups * 256 in all.  flops = 2 * 64 lanes * 63 * iters * 4 * workgroups for patterns
 * 0-2, 4 and 5 and 4096 * 4 * iters * 4 * workgroups for pattern 3.  Asynchronous on the given stream.
 */
st_status st_probe_issue_rate(int pattern, int workgroups, int iters, float *out, void *hip_stream);

/* Static, NUL-terminated description of a status value. */
const char *st_status_str(st_status status);

/* Library version, "major.minor". */
const char *st_conv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ST_CONV_H */
