"""Pins for the CPU oracle: every check here is fixed by the paper or by mathematics,
none by the oracle itself and none by the GPU path.

Citations are to SparseTrain (arXiv 1911.10175): Eq. (1) and the passage after Eq. (2)
in Sec. 2.1 (definitions of FWD, BWI, BWW), Sec. 3.3 (stride-1 BWI is FWD with transposed
filters), Sec. 5.2 (a 1x1 output is a weighted sum of the input channels at that pixel),
Alg. 1 and Alg. 4 (input-stationary forms with the zero test).
"""
import os

import numpy as np
import pytest
import torch

from oracle import st_ref
from oracle.st_ref import Geom

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(1234)


def rand(shape, zero_frac=0.0):
    a = RNG.standard_normal(shape).astype(np.float32)
    if zero_frac > 0:
        a[RNG.random(shape) < zero_frac] = 0.0
    return a


# ---------------------------------------------------------------------------
# brute force on explicitly padded arrays, written independently of the oracle
# ---------------------------------------------------------------------------
def brute_fwd(g: Geom, x, w):
    xp = np.zeros((g.N, g.C, g.H + 2 * g.pad_h, g.W + 2 * g.pad_w), dtype=np.float64)
    xp[:, :, g.pad_h:g.pad_h + g.H, g.pad_w:g.pad_w + g.W] = x
    y = np.zeros(g.y_shape, dtype=np.float64)
    for i in range(g.N):
        for k in range(g.K):
            for yy in range(g.OH):
                for xx in range(g.OW):
                    acc = 0.0
                    for c in range(g.C):
                        for v in range(g.S):
                            for u in range(g.R):
                                acc += xp[i, c, yy * g.stride_h + v, xx * g.stride_w + u] * float(w[k, c, v, u])
                    y[i, k, yy, xx] = acc
    return y


def brute_bwi(g: Geom, dy, w):
    """d/dx of sum(y*dy): spread every dy element over the padded input it read, then crop."""
    dxp = np.zeros((g.N, g.C, g.H + 2 * g.pad_h, g.W + 2 * g.pad_w), dtype=np.float64)
    for i in range(g.N):
        for k in range(g.K):
            for yy in range(g.OH):
                for xx in range(g.OW):
                    for c in range(g.C):
                        for v in range(g.S):
                            for u in range(g.R):
                                dxp[i, c, yy * g.stride_h + v, xx * g.stride_w + u] += \
                                    float(dy[i, k, yy, xx]) * float(w[k, c, v, u])
    return dxp[:, :, g.pad_h:g.pad_h + g.H, g.pad_w:g.pad_w + g.W]


def brute_bww(g: Geom, x, dy):
    xp = np.zeros((g.N, g.C, g.H + 2 * g.pad_h, g.W + 2 * g.pad_w), dtype=np.float64)
    xp[:, :, g.pad_h:g.pad_h + g.H, g.pad_w:g.pad_w + g.W] = x
    dw = np.zeros(g.w_shape, dtype=np.float64)
    for k in range(g.K):
        for c in range(g.C):
            for v in range(g.S):
                for u in range(g.R):
                    acc = 0.0
                    for i in range(g.N):
                        for yy in range(g.OH):
                            for xx in range(g.OW):
                                acc += xp[i, c, yy * g.stride_h + v, xx * g.stride_w + u] * float(dy[i, k, yy, xx])
                    dw[k, c, v, u] = acc
    return dw


TINY_GEOMS = [
    Geom(2, 3, 4, 5, 7, 3, 2, 1, 1, 1, 0),     # non-square everything, pad_w != pad_h
    Geom(1, 2, 3, 6, 5, 2, 3, 2, 1, 0, 1),     # stride_w = 2
    Geom(2, 2, 2, 7, 6, 3, 3, 2, 2, 1, 1),     # stride 2 both, 3x3 pad 1
    Geom(1, 3, 2, 4, 4, 1, 1, 1, 1, 0, 0),     # 1x1
    Geom(1, 1, 1, 5, 6, 3, 3, 1, 2, 2, 1),     # pad larger than needed, stride_h = 2
    Geom(1, 2, 2, 3, 3, 5, 5, 1, 1, 2, 2),     # filter larger than image interior
]


@pytest.mark.parametrize("g", TINY_GEOMS, ids=lambda g: f"{g.N}x{g.C}x{g.K}_{g.H}x{g.W}_{g.S}x{g.R}")
def test_brute_force_all_passes(g):
    x = rand(g.x_shape, 0.4)
    w = rand(g.w_shape)
    dy = rand(g.y_shape, 0.4)
    y, y_abs = st_ref.conv_fwd(g, x, w)
    np.testing.assert_allclose(y, brute_fwd(g, x, w), rtol=0, atol=1e-12)
    np.testing.assert_allclose(y_abs, brute_fwd(g, np.abs(x), np.abs(w)), rtol=0, atol=1e-12)
    dx, dx_abs = st_ref.conv_bwi(g, dy, w)
    np.testing.assert_allclose(dx, brute_bwi(g, dy, w), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dx_abs, brute_bwi(g, np.abs(dy), np.abs(w)), rtol=0, atol=1e-12)
    dw, dw_abs = st_ref.conv_bww(g, x, dy)
    np.testing.assert_allclose(dw, brute_bww(g, x, dy), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dw_abs, brute_bww(g, np.abs(x), np.abs(dy)), rtol=0, atol=1e-12)


def _read_golden(path):
    blocks = {}
    with open(path) as f:
        lines = [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]
    i = 0
    while i < len(lines):
        head = lines[i].split()
        name, shape = head[0], tuple(int(t) for t in head[1:])
        need = int(np.prod(shape))
        vals = []
        i += 1
        while len(vals) < need:
            vals += [float(t) for t in lines[i].split()]
            i += 1
        blocks[name] = np.array(vals).reshape(shape)
    return blocks


def test_hand_worked_eq1():
    """Eq. (1) on a 2-channel 3x4 image with a 2x3 filter, worked by hand in the fixture."""
    b = _read_golden(os.path.join(GOLDEN, "eq1_worked_example.txt"))
    g = Geom(1, 2, 1, 3, 4, R=3, S=2)
    y, y_abs = st_ref.conv_fwd(g, b["x"].astype(np.float32), b["w"].astype(np.float32))
    np.testing.assert_array_equal(y, b["y"])
    np.testing.assert_array_equal(y_abs, b["abs"])


def test_table2_skippable_fma_counts():
    """T = R*Q/V (Sec. 3.2.2/3.2.3, Table 2; Sec. 5.1-5.2): the number of FMAs the
    input-stationary loop issues per non-zero input element and K-tile, counted by running
    Alg. 1 on a one-hot input and dividing by the vector length."""
    rows = np.loadtxt(os.path.join(GOLDEN, "table2_skippable.txt"), comments="#", dtype=int)
    for R, Q, V, T in rows:
        assert R * Q // V == T
        # a single interior non-zero input element with K = Q output channels touches R outputs per
        # filter row; count the non-zero outputs of the scatter form for S = 1
        g = Geom(1, 1, int(Q), 1, 2 * int(R) + 1, int(R), 1, 1, 1, int(R) - 1, 0)
        x = np.zeros(g.x_shape, dtype=np.float32)
        x[0, 0, 0, R] = 1.0
        w = np.ones(g.w_shape, dtype=np.float32)
        y, skipped = st_ref.conv_fwd_scatter(g, x, w)
        assert np.count_nonzero(y) // V == T
        assert skipped == g.W - 1


# ---------------------------------------------------------------------------
# closed forms
# ---------------------------------------------------------------------------
def test_all_ones_counts_taps():
    """x = 1, w = 1: every output equals C times the number of taps that fall inside the image."""
    g = Geom(1, 5, 2, 6, 9, 3, 3, 1, 1, 1, 1)
    y, y_abs = st_ref.conv_fwd(g, np.ones(g.x_shape, np.float32), np.ones(g.w_shape, np.float32))
    exp = np.full((g.OH, g.OW), 9.0)
    exp[0, :] = exp[-1, :] = 6.0
    exp[:, 0] = exp[:, -1] = 6.0
    exp[0, 0] = exp[0, -1] = exp[-1, 0] = exp[-1, -1] = 4.0
    for k in range(g.K):
        np.testing.assert_array_equal(y[0, k], g.C * exp)
    np.testing.assert_array_equal(y, y_abs)
    # BWW of all-ones: dw[v,u] = N * number of output pixels whose tap (v,u) is in range
    dw, _ = st_ref.conv_bww(g, np.ones(g.x_shape, np.float32), np.ones(g.y_shape, np.float32))
    cnt_h = np.array([g.OH - 1, g.OH, g.OH - 1], dtype=float)
    cnt_w = np.array([g.OW - 1, g.OW, g.OW - 1], dtype=float)
    np.testing.assert_array_equal(dw[1, 3], np.outer(cnt_h, cnt_w))
    # BWI of all-ones: dx = K * number of outputs that read the pixel
    dx, _ = st_ref.conv_bwi(g, np.ones(g.y_shape, np.float32), np.ones(g.w_shape, np.float32))
    np.testing.assert_array_equal(dx[0, 0], g.K * exp)


def test_identity_filter_and_zero_input():
    g = Geom(2, 4, 4, 5, 6, 3, 3, 1, 1, 1, 1)
    x = rand(g.x_shape)
    w = np.zeros(g.w_shape, np.float32)
    for c in range(g.C):
        w[c, c, 1, 1] = 1.0
    y, _ = st_ref.conv_fwd(g, x, w)
    np.testing.assert_array_equal(y, x.astype(np.float64))
    y0, a0 = st_ref.conv_fwd(g, np.zeros(g.x_shape, np.float32), rand(g.w_shape))
    assert not y0.any() and not a0.any()


def test_shifted_delta_filter_direction():
    """A filter that is 1 at tap (v=0,u=2) makes y[oh,ow] = x[oh-pad+0, ow-pad+2]: fixes the tap
    orientation (correlation, no flip) and which filter axis pairs with which image axis."""
    g = Geom(1, 1, 1, 5, 6, 3, 3, 1, 1, 1, 1)
    x = rand(g.x_shape)
    w = np.zeros(g.w_shape, np.float32)
    w[0, 0, 0, 2] = 1.0
    y, _ = st_ref.conv_fwd(g, x, w)
    exp = np.zeros((5, 6))
    exp[1:, :-1] = x[0, 0, :-1, 1:]
    np.testing.assert_array_equal(y[0, 0], exp)


def test_one_by_one_is_matrix_product():
    g = Geom(3, 7, 5, 4, 6, 1, 1)
    x, w = rand(g.x_shape, 0.3), rand(g.w_shape)
    y, _ = st_ref.conv_fwd(g, x, w)
    exp = np.einsum("kc,nchw->nkhw", w[:, :, 0, 0].astype(np.float64), x.astype(np.float64))
    np.testing.assert_allclose(y, exp, rtol=0, atol=1e-12)
    dy = rand(g.y_shape, 0.3)
    dx, _ = st_ref.conv_bwi(g, dy, w)
    np.testing.assert_allclose(dx, np.einsum("kc,nkhw->nchw", w[:, :, 0, 0].astype(np.float64),
                                             dy.astype(np.float64)), rtol=0, atol=1e-12)
    dw, _ = st_ref.conv_bww(g, x, dy)
    np.testing.assert_allclose(dw[:, :, 0, 0], np.einsum("nkhw,nchw->kc", dy.astype(np.float64),
                                                         x.astype(np.float64)), rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------
# library routine (CPU fp64 convolution and its autograd), used only to check the oracle
# ---------------------------------------------------------------------------
LIB_GEOMS = [
    Geom(2, 16, 16, 8, 8, 3, 3, 1, 1, 1, 1),
    Geom(2, 5, 6, 9, 11, 3, 5, 1, 1, 1, 2),      # R=3 wide, S=5 tall
    Geom(2, 4, 6, 10, 9, 3, 3, 2, 2, 1, 1),
    Geom(1, 8, 4, 7, 7, 1, 1, 1, 1, 0, 0),
    Geom(1, 3, 3, 8, 10, 5, 3, 2, 1, 2, 0),
]


@pytest.mark.parametrize("g", LIB_GEOMS, ids=lambda g: f"{g.C}to{g.K}_{g.H}x{g.W}_{g.S}x{g.R}_s{g.stride_h}{g.stride_w}")
def test_against_library_conv(g):
    x, w, dy = rand(g.x_shape, 0.5), rand(g.w_shape), rand(g.y_shape, 0.5)
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.conv2d(xt, wt, stride=(g.stride_h, g.stride_w), padding=(g.pad_h, g.pad_w))
    assert tuple(yt.shape) == g.y_shape
    yt.backward(torch.tensor(dy, dtype=torch.float64))
    y, _ = st_ref.conv_fwd(g, x, w)
    dx, _ = st_ref.conv_bwi(g, dy, w)
    dw, _ = st_ref.conv_bww(g, x, dy)
    np.testing.assert_allclose(y, yt.detach().numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=0, atol=1e-11)


# ---------------------------------------------------------------------------
# identities
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("g", LIB_GEOMS + TINY_GEOMS[:3], ids=lambda g: f"{g.C}to{g.K}_{g.H}x{g.W}_{g.S}x{g.R}")
def test_adjoint_identities(g):
    x, w, dy = rand(g.x_shape, 0.5), rand(g.w_shape), rand(g.y_shape, 0.5)
    y, _ = st_ref.conv_fwd(g, x, w)
    dx, _ = st_ref.conv_bwi(g, dy, w)
    dw, _ = st_ref.conv_bww(g, x, dy)
    a = float(np.sum(y * dy))
    b = float(np.sum(x.astype(np.float64) * dx))
    c = float(np.sum(w.astype(np.float64) * dw))
    scale = float(np.sum(np.abs(y * dy))) + 1e-300
    assert abs(a - b) / scale < 1e-12
    assert abs(a - c) / scale < 1e-12


def test_stride1_bwi_is_fwd_with_rotated_transposed_filters():
    """Sec. 3.3: for unit stride BWI equals FWD on dy with the filters transposed (channel roles
    swapped, taps reversed) and padding (S-1-pad_h, R-1-pad_w)."""
    g = Geom(2, 6, 4, 7, 9, 3, 5, 1, 1, 1, 2)
    dy, w = rand(g.y_shape, 0.4), rand(g.w_shape)
    dx, dx_abs = st_ref.conv_bwi(g, dy, w)
    wt = np.ascontiguousarray(w.transpose(1, 0, 2, 3)[:, :, ::-1, ::-1])
    g2 = Geom(g.N, g.K, g.C, g.OH, g.OW, g.R, g.S, 1, 1, g.R - 1 - g.pad_w, g.S - 1 - g.pad_h)
    assert (g2.OH, g2.OW) == (g.H, g.W)
    y2, y2_abs = st_ref.conv_fwd(g2, dy, wt)
    np.testing.assert_allclose(dx, y2, rtol=0, atol=1e-12)
    np.testing.assert_allclose(dx_abs, y2_abs, rtol=0, atol=1e-12)


@pytest.mark.parametrize("g", LIB_GEOMS + TINY_GEOMS, ids=lambda g: f"{g.C}to{g.K}_{g.H}x{g.W}_{g.S}x{g.R}_s{g.stride_h}{g.stride_w}")
def test_scatter_forms_equal_definition(g):
    """Alg. 1 / its BWI twin / Alg. 4 (both tested operands) reach the dense result, and
    skip exactly the zero elements of the tested operand."""
    for zf in (0.0, 0.6, 1.0):
        x, w, dy = rand(g.x_shape, zf), rand(g.w_shape), rand(g.y_shape, zf)
        y, _ = st_ref.conv_fwd(g, x, w)
        ys, sk = st_ref.conv_fwd_scatter(g, x, w)
        np.testing.assert_allclose(ys, y, rtol=0, atol=1e-11)
        assert sk == np.count_nonzero(x == 0)
        dx, _ = st_ref.conv_bwi(g, dy, w)
        dxs, sk = st_ref.conv_bwi_scatter(g, dy, w)
        np.testing.assert_allclose(dxs, dx, rtol=0, atol=1e-11)
        assert sk == np.count_nonzero(dy == 0)
        dw, _ = st_ref.conv_bww(g, x, dy)
        for test_dy in (False, True):
            dws, sk = st_ref.conv_bww_scatter(g, x, dy, test_dy)
            np.testing.assert_allclose(dws, dw, rtol=0, atol=1e-11)
            assert sk == np.count_nonzero((dy if test_dy else x) == 0)


def test_zero_semantics_negative_zero_and_denormal():
    """The zero test is a float compare against 0 (Alg. 3): -0.0 is skipped, a denormal is not."""
    g = Geom(1, 1, 1, 1, 4, 1, 1)
    x = np.array([0.0, -0.0, 1e-45, 2.0], dtype=np.float32).reshape(g.x_shape)
    assert x[0, 0, 0, 2] != 0 and np.signbit(x[0, 0, 0, 1])
    w = np.full(g.w_shape, 3.0, np.float32)
    ys, skipped = st_ref.conv_fwd_scatter(g, x, w)
    assert skipped == 2
    y, _ = st_ref.conv_fwd(g, x, w)
    np.testing.assert_array_equal(ys, y)
    assert y[0, 0, 0, 2] == float(np.float32(1e-45)) * 3.0 and y[0, 0, 0, 2] > 0


def test_sampled_forms_match_full():
    g = Geom(2, 6, 5, 7, 8, 3, 3, 1, 1, 1, 1)
    x, w, dy = rand(g.x_shape, 0.5), rand(g.w_shape), rand(g.y_shape, 0.5)
    y, ya = st_ref.conv_fwd(g, x, w)
    dx, dxa = st_ref.conv_bwi(g, dy, w)
    dw, dwa = st_ref.conv_bww(g, x, dy)
    for full, full_abs, fn, a, b, shape in ((y, ya, st_ref.conv_fwd_at, x, w, g.y_shape),
                                            (dx, dxa, st_ref.conv_bwi_at, dy, w, g.x_shape),
                                            (dw, dwa, st_ref.conv_bww_at, x, dy, g.w_shape)):
        coords = np.stack([RNG.integers(0, s, 50) for s in shape], axis=1).astype(np.int32)
        out, out_abs = fn(g, a, b, coords)
        np.testing.assert_array_equal(out, full[tuple(coords.T)])
        np.testing.assert_array_equal(out_abs, full_abs[tuple(coords.T)])
    with pytest.raises(ValueError):
        st_ref.conv_fwd_at(g, x, w, np.array([[0, 0, 7, 0]], dtype=np.int32))


def test_bad_geometry_rejected():
    with pytest.raises(ValueError):
        st_ref.conv_fwd(Geom(1, 1, 1, 2, 2, 3, 3), np.zeros((1, 1, 2, 2), np.float32),
                        np.zeros((1, 1, 3, 3), np.float32))


# ---------------------------------------------------------------------------
# planted mistakes: each pin above must be able to see a plausible error.  The mistakes are
# planted in a copy of the definition written here (on the CPU), never in the oracle.
# ---------------------------------------------------------------------------
def _variant_fwd(g, x, w, flip=False, swap_rs=False, drop_pad=False):
    xp = np.zeros((g.N, g.C, g.H + 2 * g.pad_h, g.W + 2 * g.pad_w))
    xp[:, :, g.pad_h:g.pad_h + g.H, g.pad_w:g.pad_w + g.W] = x
    y = np.zeros(g.y_shape)
    for yy in range(g.OH):
        for xx in range(g.OW):
            for v in range(g.S):
                for u in range(g.R):
                    vv, uu = (g.S - 1 - v, g.R - 1 - u) if flip else (v, u)
                    if swap_rs and g.R == g.S:
                        vv, uu = uu, vv
                    ih, iw = yy * g.stride_h + v, xx * g.stride_w + u
                    if drop_pad:
                        ih, iw = min(ih + g.pad_h, xp.shape[2] - 1), min(iw + g.pad_w, xp.shape[3] - 1)
                    y[:, :, yy, xx] += np.einsum("nc,kc->nk", xp[:, :, ih, iw], w[:, :, vv, uu].astype(np.float64))
    return y


def test_pins_detect_planted_mistakes():
    g = Geom(2, 3, 4, 6, 7, 3, 3, 1, 1, 1, 1)
    x, w = rand(g.x_shape), rand(g.w_shape)
    y, _ = st_ref.conv_fwd(g, x, w)
    assert np.allclose(_variant_fwd(g, x, w), y, atol=1e-10)
    assert not np.allclose(_variant_fwd(g, x, w, flip=True), y, atol=1e-3)
    assert not np.allclose(_variant_fwd(g, x, w, swap_rs=True), y, atol=1e-3)
    assert not np.allclose(_variant_fwd(g, x, w, drop_pad=True), y, atol=1e-3)


# ---------------------------------------------------------------------------
# the checker itself: every GPU verdict goes through st_ref.rel_err, so it is pinned by cases
# worked by hand and by deviations planted here (never in the oracle's convolutions)
# ---------------------------------------------------------------------------
def test_rel_err_hand_computed():
    ref = np.array([1.0, 2.0, -3.0, 0.0])
    scale = np.array([2.0, 4.0, 3.0, 0.0])
    assert st_ref.rel_err(ref.copy(), ref, scale) == (0.0, 0)
    got = np.array([1.5, 2.0, -3.0, 0.0])           # |1.5 - 1| / 2
    assert st_ref.rel_err(got, ref, scale) == (0.25, 0)
    got = np.array([1.0, 2.0, 3.0, -0.0])           # sign flipped: |3 + 3| / 3; -0 is a zero
    assert st_ref.rel_err(got, ref, scale) == (2.0, 0)
    got = np.array([1.0, 2.0, -3.0, 1e-30])         # all terms zero, value not zero
    assert st_ref.rel_err(got, ref, scale) == (0.0, 1)


def test_rel_err_is_per_element_not_global():
    """A deviation is measured against the scale of its own element: a large neighbour hides nothing."""
    ref = np.array([1e6, 1e-3])
    scale = np.array([2e6, 2e-3])
    got = np.array([1e6, 1e-3 + 2e-3 * 3e-4])
    err, bad = st_ref.rel_err(got, ref, scale)
    assert bad == 0 and err == pytest.approx(3e-4, rel=1e-9)


def test_rel_err_flags_planted_deviation_on_a_real_layer():
    """One element of an fp32 copy of the oracle's result moved by 2e-4 of its scale must be reported
    at that size (the GPU tests' bar is 1e-4), one moved by 0.5e-4 must pass, and the unperturbed
    copy stays at fp32 rounding."""
    g = Geom(2, 16, 16, 6, 7, 3, 3, 1, 1, 1, 1)
    x, w = rand(g.x_shape, 0.5), rand(g.w_shape)
    y, ya = st_ref.conv_fwd(g, x, w)
    got = y.astype(np.float32)
    err0, bad0 = st_ref.rel_err(got, y, ya)
    assert bad0 == 0 and err0 < 2.0 ** -23
    idx = (1, 5, 3, 2)
    assert ya[idx] > 0
    for rel, must_pass in ((2e-4, False), (0.5e-4, True)):
        bent = got.astype(np.float64)
        bent[idx] = y[idx] + rel * ya[idx]
        err, bad = st_ref.rel_err(bent, y, ya)
        assert bad == 0 and err == pytest.approx(rel, rel=1e-6)
        assert (err <= 1e-4) == must_pass


def test_rel_err_flags_non_finite_and_unwritten_zero_rows():
    g = Geom(1, 16, 16, 4, 4, 3, 3, 1, 1, 1, 1)
    x, w = rand(g.x_shape), rand(g.w_shape)
    x[0, :, :, :] = 0.0                                  # every term of every output is zero
    y, ya = st_ref.conv_fwd(g, x, w)
    assert not ya.any() and not y.any()
    got = np.zeros_like(y)
    assert st_ref.rel_err(got, y, ya) == (0.0, 0)
    got[0, 3, 1, 1] = 1e-20
    got[0, 4, 2, 2] = np.nan
    assert st_ref.rel_err(got, y, ya) == (0.0, 2)
    x2 = rand(g.x_shape)
    y2, ya2 = st_ref.conv_fwd(g, x2, w)
    bent = y2.copy()
    bent[0, 0, 0, 0] = np.nan
    err, _ = st_ref.rel_err(bent, y2, ya2)
    assert err == float("inf")
    bent[0, 0, 0, 0] = np.inf
    assert st_ref.rel_err(bent, y2, ya2)[0] == float("inf")
    with pytest.raises(ValueError):
        st_ref.rel_err(y2[:, :1], y2, ya2)
