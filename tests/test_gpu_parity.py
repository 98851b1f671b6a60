"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Every test here needs an MI355X."""
import numpy as np
import pytest
import torch

import stgen
from oracle import st_ref
from oracle.st_ref import Geom

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from tests.gpu_harness import (DeviceLayer, assert_close, check_all_passes_full,
                                   check_all_passes_sampled, desc_of, gather_activations, sample_coords)
    import paper_1911_10175_amd as st


def geom_of(layer: stgen.Layer) -> Geom:
    return Geom(layer.N, layer.C, layer.K, layer.H, layer.W, layer.R, layer.S,
                layer.stride, layer.stride, layer.pad, layer.pad)


def synth(g: Geom, p_x, p_dy, seed):
    x = stgen.relu_sparse(g.x_shape, p_x, 4 * seed)
    w = stgen.he_normal(g.w_shape, 4 * seed + 1)
    dy = stgen.bernoulli_masked(g.y_shape, p_dy, 4 * seed + 2, 4 * seed + 3)
    return x, w, dy


def test_library_is_the_hip_build():
    assert st.lib_path().endswith("libst_conv.so")
    assert st.st_conv_version()


def test_issue_rate_probe_runs():
    """The measurement aid of bench.py --probe-valu: every pattern launches and stores its result word
    (the vector streams start from zeroed registers, so their words are 0; the matrix stream's are finite)."""
    out = torch.full((8 * 256,), float("nan"), device="cuda")
    for pattern in range(6):
        out.fill_(float("nan"))
        st.st_probe_issue_rate(pattern, 8, 3, out)
        torch.cuda.synchronize()
        assert bool((out == 0).all()) if pattern != 3 else bool(torch.isfinite(out).all()), pattern


def test_config1_tiny_layer():
    """N=1, C=K=16, 8x8, 3x3 pad 1, x 50 % zeros, dy = g * (FWD output > 0), seed 0."""
    L = stgen.TINY
    g = geom_of(L)
    x, w, _ = stgen.make_layer_tensors(L, seed=0)
    y_ref, _ = st_ref.conv_fwd(g, x, w)
    dy = stgen.relu_grad(y_ref.astype(np.float32), 2)
    assert 0.3 < stgen.zero_fraction(x) < 0.7 and 0.2 < stgen.zero_fraction(dy) < 0.8
    check_all_passes_full(g, x, w, dy, "config1")


SMALL = [
    # several 8x8 tiles with a ragged tail in both directions
    ("3x3_ragged", Geom(2, 32, 64, 13, 19, 3, 3, 1, 1, 1, 1), 0.5, 0.5),
    # 128 output channels per wavefront, 3 channel blocks
    ("3x3_k128", Geom(2, 48, 128, 20, 20, 3, 3, 1, 1, 1, 1), 0.6, 0.45),
    ("3x3_k256_c64", Geom(1, 64, 256, 9, 17, 3, 3, 1, 1, 1, 1), 0.3, 0.7),
    # fewer channels than lanes
    ("3x3_k16", Geom(3, 16, 16, 10, 7, 3, 3, 1, 1, 1, 1), 0.5, 0.5),
    ("3x3_k48_c80", Geom(1, 80, 48, 11, 12, 3, 3, 1, 1, 1, 1), 0.5, 0.5),
    # channel split across the wavefronts of a workgroup: 2 shares (6 channel blocks), 4 shares
    ("3x3_c96_split2", Geom(1, 96, 128, 9, 9, 3, 3, 1, 1, 1, 1), 0.5, 0.5),
    ("3x3_c64_k64_split4", Geom(2, 64, 64, 10, 13, 3, 3, 1, 1, 1, 1), 0.5, 0.5),
    ("3x3_c256_k128_split4", Geom(1, 256, 128, 6, 7, 3, 3, 1, 1, 1, 1), 0.6, 0.6),
    # 8 and 16 shares (launches with few tasks): FWD reduces C, BWI reduces K; two- and one-channel-per-lane tiles
    ("3x3_c128_k256_split8", Geom(2, 128, 256, 9, 10, 3, 3, 1, 1, 1, 1), 0.5, 0.5),
    ("3x3_c384_k64_split8", Geom(1, 384, 64, 7, 7, 3, 3, 1, 1, 1, 1), 0.5, 0.6),
    ("3x3_c512_k256_split16", Geom(1, 512, 256, 5, 9, 3, 3, 1, 1, 1, 1), 0.6, 0.5),
    ("3x3_c256_k64_split16_pad2", Geom(2, 256, 64, 6, 6, 3, 3, 1, 1, 2, 2), 0.5, 0.5),
    # other paddings of the 3x3 fast path
    ("3x3_pad0", Geom(2, 32, 64, 12, 14, 3, 3, 1, 1, 0, 0), 0.5, 0.5),
    ("3x3_pad2_1", Geom(1, 32, 64, 9, 10, 3, 3, 1, 1, 2, 1), 0.5, 0.5),
    # 1x1
    ("1x1_k128", Geom(2, 64, 128, 12, 12, 1, 1), 0.4, 0.5),
    ("1x1_k64", Geom(2, 256, 64, 9, 11, 1, 1), 0.55, 0.5),
    # channel counts that are no multiple of the 32-wide MFMA blocks or of the 64 lanes, ragged last pixel chunk
    ("1x1_k48_c80", Geom(3, 80, 48, 7, 5, 1, 1), 0.5, 0.5),
    ("1x1_k16_c16", Geom(1, 16, 16, 3, 3, 1, 1), 0.5, 0.5),
    ("1x1_k208_c96", Geom(2, 96, 208, 14, 14, 1, 1), 0.4, 0.6),
    ("1x1_k512_c32", Geom(1, 32, 512, 6, 6, 1, 1), 0.5, 0.5),
    ("3x3_stride2", Geom(2, 32, 32, 14, 14, 3, 3, 2, 2, 1, 1), 0.5, 0.5),
    # shapes only the generic kernels cover
    ("5x5_pad2", Geom(1, 16, 32, 9, 9, 5, 5, 1, 1, 2, 2), 0.5, 0.5),
    ("r3_s1_stride_1x2", Geom(1, 32, 16, 8, 11, 3, 1, 2, 1, 1, 0), 0.5, 0.5),
    ("1x1_stride2", Geom(1, 32, 32, 9, 9, 1, 1, 2, 2, 0, 0), 0.5, 0.5),
]


@pytest.mark.parametrize("label,g,px,pdy", SMALL, ids=[s[0] for s in SMALL])
def test_small_shapes_all_passes(label, g, px, pdy):
    x, w, dy = synth(g, px, pdy, seed=3)
    check_all_passes_full(g, x, w, dy, label)


# the dense 1x1 form that keeps the filter matrix in LDS: every instance (64 / 128 / 256 produced channels, channel
# loops of 4, 8 and 16 blocks, i.e. both prefetch depths), FWD and BWI, with 8268 pixels: 258 whole tiles of 32 and
# one of 12, spread over 256 workgroups so that some get two tiles and the last ones none
PW_LDS = [Geom(3, 256, 64, 53, 52, 1, 1), Geom(3, 64, 256, 53, 52, 1, 1), Geom(3, 64, 64, 53, 52, 1, 1),
          Geom(3, 128, 128, 53, 52, 1, 1), Geom(3, 64, 128, 53, 52, 1, 1), Geom(12, 128, 64, 56, 56, 1, 1)]


@pytest.mark.parametrize("g", PW_LDS, ids=[f"{g.C}to{g.K}_n{g.N}" for g in PW_LDS])
def test_dense_1x1_with_filters_in_lds(g):
    x, w, dy = synth(g, 0.5, 0.5, seed=29)
    check_all_passes_full(g, x, w, dy, f"1x1 {g.C}->{g.K}", passes=("fwd", "bwi"), variants=(True,))


@pytest.mark.parametrize("p", [0.0, 0.9, 1.0])
def test_degenerate_sparsity(p):
    """Fully dense, very sparse and all-zero tested operands."""
    g = Geom(2, 32, 128, 11, 13, 3, 3, 1, 1, 1, 1)
    x, w, dy = synth(g, min(p, 0.9), min(p, 0.9), seed=5)
    if p == 1.0:
        x[:] = 0.0
        dy[:] = 0.0
    check_all_passes_full(g, x, w, dy, f"p={p}")


def test_zero_semantics_on_gpu():
    """-0.0 is skipped like +0.0, denormals are not flushed before the test: a denormal input
    times a huge filter value must survive in the sparse result as in the oracle."""
    g = Geom(1, 16, 16, 8, 8, 3, 3, 1, 1, 1, 1)
    x = np.zeros(g.x_shape, np.float32)
    x[0, :, ::2, ::2] = -0.0
    x[0, 3, 4, 4] = 1e-40            # denormal
    x[0, 5, 1, 6] = 2.0
    w = np.full(g.w_shape, 1e30, np.float32)
    dy = np.zeros(g.y_shape, np.float32)
    dy[0, 2, 3, 3] = -0.0
    dy[0, 7, 5, 2] = 1e-40
    check_all_passes_full(g, x, w, dy, "zero-semantics", passes=("fwd", "bwi"))
    L = DeviceLayer(g, x, w, dy)
    y = L.fwd(False)
    assert y[0, 0, 4, 4] > 0                     # the denormal contributed


def test_sparse_equals_dense_control_and_is_deterministic():
    g = Geom(2, 64, 128, 16, 16, 3, 3, 1, 1, 1, 1)
    x, w, dy = synth(g, 0.5, 0.5, seed=9)
    L = DeviceLayer(g, x, w, dy)
    for fn in (L.fwd, L.bwi, L.bww):
        a, b = fn(False), fn(False)
        assert np.array_equal(a, b), "two runs of the sparse kernel differ"
        c = fn(True)
        assert np.allclose(a, c, rtol=1e-3, atol=1e-4)


@pytest.mark.parametrize("cs,ch", [(1, 48), (2, 96), (4, 64), (8, 128), (16, 256)])
def test_fwd_bwi_channel_split(cs, ch):
    """Every channel split of the zero-skipping FWD / BWI kernel gives the oracle's result on ragged
    tiles.  The split follows from the descriptor alone: with C = K = ch and this few tiles a task is
    shared by the largest power of two <= 16 that divides ch / 16 wavefronts, each reducing that share
    of the input channels (1 for 3 blocks, 2 for 6, 4 for 4, 8 for 8, 16 for 16)."""
    g = Geom(2, ch, ch, 10, 13, 3, 3, 1, 1, 1, 1)
    assert (ch // 16) % cs == 0 and (cs == 16 or (ch // 16) % (2 * cs) != 0)
    x, w, dy = synth(g, 0.6, 0.5, seed=31 + cs)
    check_all_passes_full(g, x, w, dy, f"split {cs}", passes=("fwd", "bwi"), variants=(False,))


BWW_DY_SHAPES = [
    ("3x3 pad0 C<K", Geom(2, 32, 80, 13, 19, 3, 3, 1, 1, 0, 0)),
    ("3x3 pad2 C>K", Geom(2, 144, 48, 9, 12, 3, 3, 1, 1, 2, 2)),
    ("3x3 pad(1,0)", Geom(3, 64, 64, 17, 8, 3, 3, 1, 1, 1, 0)),
    ("1x1", Geom(2, 96, 208, 14, 14, 1, 1, 1, 1, 0, 0)),
    ("3x3 stride2 (generic)", Geom(2, 32, 48, 15, 15, 3, 3, 2, 2, 1, 1)),
    ("5x5 (generic)", Geom(1, 16, 32, 9, 9, 5, 5, 1, 1, 2, 2)),
]


@pytest.mark.parametrize("label,g", BWW_DY_SHAPES, ids=[s[0] for s in BWW_DY_SHAPES])
@pytest.mark.parametrize("px,pdy", [(0.0, 0.9), (0.6, 0.5)])
def test_bww_dy_tested_operand(label, g, px, pdy):
    """BWW with the zero test on dy (Sec. 3.4, closing remark): same tensor as the x-testing form."""
    x, w, dy = synth(g, px, pdy, seed=31)
    L = DeviceLayer(g, x, w, dy)
    ref, ref_abs = st_ref.conv_bww(g, x, dy)
    got = L.bww("dy")
    assert_close(got, ref, ref_abs, f"{label} BWW tests dy")
    assert np.array_equal(got, L.bww("dy")), "two runs differ"


def test_bww_dy_skips_on_dy_only():
    """All-zero dy with non-finite-free x gives exactly zero; -0 in dy is skipped, a denormal is kept."""
    g = Geom(1, 16, 16, 8, 8, 3, 3, 1, 1, 1, 1)
    x = np.full(g.x_shape, 1e30, np.float32)
    dy = np.zeros(g.y_shape, np.float32)
    dy[0, :, ::2, ::2] = -0.0
    L = DeviceLayer(g, x, None, dy)
    assert not L.bww("dy").any()
    dy[0, 7, 5, 2] = 1e-40
    L = DeviceLayer(g, x, None, dy)
    ref, ref_abs = st_ref.conv_bww(g, x, dy)
    got = L.bww("dy")
    assert_close(got, ref, ref_abs, "denormal dy")
    assert got[7, 0, 1, 1] > 0


STRIDE2 = [
    ("s2 32->128 @32", Geom(2, 32, 128, 32, 32, 3, 3, 2, 2, 1, 1)),          # FWD wide 4x8; BWI narrow 8x8
    ("s2 128->48 @28", Geom(2, 128, 48, 28, 28, 3, 3, 2, 2, 1, 1)),          # FWD narrow 4x7; BWI wide 2x14
    ("s2 128->128 30x26", Geom(1, 128, 128, 30, 26, 3, 3, 2, 2, 1, 1)),      # ragged tiles everywhere
    ("s2 48->32 @14", Geom(2, 48, 32, 14, 14, 3, 3, 2, 2, 1, 1)),            # FWD narrow 4x7; BWI narrow 4x14
    ("s2 64->64 15x17", Geom(1, 64, 64, 15, 17, 3, 3, 2, 2, 1, 1)),          # odd image sizes
    ("s2 pad0", Geom(2, 32, 32, 17, 17, 3, 3, 2, 2, 0, 0)),                  # FWD tiled, BWI generic
    ("s2 pad2", Geom(1, 16, 128, 12, 20, 3, 3, 2, 2, 2, 2)),
    ("s2 16->16 tiny", Geom(1, 16, 16, 5, 5, 3, 3, 2, 2, 1, 1)),
    ("s2 80->48 @9x30", Geom(2, 80, 48, 9, 30, 3, 3, 2, 2, 1, 1)),
    ("s2 256->256 @28", Geom(2, 256, 256, 28, 28, 3, 3, 2, 2, 1, 1)),        # Table 1 resnet4_2/r, channel split 4
]


@pytest.mark.parametrize("label,g", STRIDE2, ids=[s[0] for s in STRIDE2])
def test_stride2_layers(label, g):
    """Stride-2 3x3 layers (Table 1, the /r rows; Sec. 3.3 on BWI with a stride)."""
    x, w, dy = synth(g, 0.5, 0.6, seed=41)
    check_all_passes_full(g, x, w, dy, label)


def test_stride2_degenerate_sparsity():
    g = Geom(1, 64, 128, 16, 16, 3, 3, 2, 2, 1, 1)
    for p in (0.0, 1.0):
        x, w, dy = synth(g, p, p, seed=43)
        if p == 1.0:
            x[:] = 0.0
            dy[:] = 0.0
        check_all_passes_full(g, x, w, dy, f"s2 p={p}")


def sampled_zero_counts(packed: np.ndarray):
    """The library's sampling recipe, restated: blocks of 1024 consecutive floats, every stride-th
    block with stride = ceil(blocks / 64) (all blocks when there are at most 64)."""
    flat = packed.reshape(-1)
    blocks = (flat.size + 1023) // 1024
    stride = (blocks + 63) // 64
    zeros = seen = 0
    for b in range(0, blocks, stride):
        chunk = flat[b * 1024:(b + 1) * 1024]
        zeros += int((chunk == 0).sum())
        seen += chunk.size
    return zeros, seen


def device_counts(ws, first_word):
    """(zeros, elements looked at) the library left in its workspace: four pairs per tensor, one per
    sampling workgroup, from word first_word on."""
    c = ws[first_word:first_word + 8].cpu().numpy().view(np.uint32).astype(np.int64)
    return int(c[0::2].sum()), int(c[1::2].sum())


@pytest.mark.parametrize("px,pdy", [(0.2, 0.8), (0.8, 0.2), (0.0, 0.0)])
@pytest.mark.parametrize("g", [Geom(2, 64, 128, 24, 24, 3, 3, 1, 1, 1, 1), Geom(4, 128, 64, 14, 14, 1, 1),
                               Geom(2, 32, 32, 16, 16, 3, 3, 2, 2, 1, 1), Geom(1, 16, 32, 9, 9, 5, 5, 1, 1, 2, 2),
                               # one tile: every form leaves a single partial sum, which the shared final sum copies
                               Geom(1, 16, 16, 8, 8, 3, 3, 1, 1, 1, 1)],
                         ids=["3x3", "1x1", "3x3s2", "5x5generic", "3x3-one-tile"])
def test_bww_auto_selects_the_sparser_operand(g, px, pdy):
    """st_conv_bww_auto: parity, and the zero counts it bases its choice on (Sec. 5.3 policy)."""
    x, w, dy = synth(g, px, pdy, seed=51)
    L = DeviceLayer(g, x, None, dy)
    ref, ref_abs = st_ref.conv_bww(g, x, dy)
    got = L.bww("auto")
    assert_close(got, ref, ref_abs, f"BWW auto px={px} pdy={pdy}")
    if g.stride_w == 2:
        # stride-2 3x3 layers: the dy-testing form is faster at any pair of sparsities and is taken unsampled
        assert np.array_equal(got, L.bww("dy"))
        return
    if g.R == 1:
        # 1x1 layers: the dense form is faster up to about 90 % zeros and is taken unsampled
        assert np.array_equal(got, L.bww(True))
        return
    zx, nx = sampled_zero_counts(st.pack_activations(x))
    zdy, ndy = sampled_zero_counts(st.pack_activations(dy))
    assert device_counts(L.auto_ws, 0) + device_counts(L.auto_ws, 8) == (zx, nx, zdy, ndy)
    # the sample agrees with the tensors' true zero fractions about which operand is sparser
    if px != pdy:
        assert (zdy * nx > zx * ndy) == (pdy > px)
    assert np.array_equal(got, L.bww("auto")), "two runs differ"
    # which form ran: the one testing the sparser operand, or, where all three forms are tiled, the dense
    # one when even that operand has fewer zeros than the break-even (25 % for 3x3)
    if g.R == 5:
        return
    best = max(px, pdy)
    form = True if best < 0.25 else ("dy" if pdy > px else False)
    assert np.array_equal(got, L.bww(form)), f"expected the form {form!r}"


@pytest.mark.parametrize("p,form", [(0.1, True), (0.9, False)])
def test_fwd_bwi_auto_pick_the_form_by_sparsity(p, form):
    """st_conv_fwd_auto / st_conv_bwi_auto: with few zeros the result is bit-identical to the dense
    entry point's, with many to the zero-skipping one's (the two sum in different orders), and the
    counters hold the zero count of the sampled blocks of the tested operand."""
    g = Geom(2, 64, 128, 24, 24, 3, 3, 1, 1, 1, 1)      # break-even of this shape: 25 % zeros
    x, w, dy = synth(g, p, p, seed=61)
    L = DeviceLayer(g, x, w, dy)
    assert not np.array_equal(L.fwd(False), L.fwd(True)), "forms indistinguishable: test is void"
    got = L.fwd("auto")
    assert device_counts(L.auto_ws, 0) == sampled_zero_counts(st.pack_activations(x))
    assert np.array_equal(got, L.fwd(form))
    got = L.bwi("auto")
    assert device_counts(L.auto_ws, 0) == sampled_zero_counts(st.pack_activations(dy))
    assert np.array_equal(got, L.bwi(form))


# one geometry per instance of the main kernel that holds both forms: (tile of the zero-skipping form, wavefronts
# per tile, tile of the dense form); minibatches large enough that the dense form does not split its channels
COMBINED = [
    (Geom(8, 64, 128, 64, 48, 3, 3, 1, 1, 1, 1), "fwd_auto_kernel<4, 8, 2, 4, 4, 8>"),
    (Geom(8, 96, 128, 64, 48, 3, 3, 1, 1, 1, 1), "fwd_auto_kernel<4, 8, 2, 2, 4, 8>"),
    (Geom(8, 64, 128, 56, 56, 3, 3, 1, 1, 1, 1), "fwd_auto_kernel<4, 7, 2, 4, 4, 8>"),
    (Geom(8, 96, 128, 56, 56, 3, 3, 1, 1, 1, 1), "fwd_auto_kernel<4, 7, 2, 2, 4, 8>"),
    (Geom(28, 64, 128, 28, 28, 3, 3, 1, 1, 1, 1), "fwd_auto_kernel<4, 7, 2, 4, 4, 28>"),
    (Geom(28, 96, 128, 28, 28, 3, 3, 1, 1, 1, 1), "fwd_auto_kernel<4, 7, 2, 2, 4, 28>"),
    (Geom(96, 64, 128, 14, 14, 3, 3, 1, 1, 1, 1), "fwd_auto_kernel<4, 7, 2, 4, 4, 14>"),
    (Geom(96, 96, 128, 14, 14, 3, 3, 1, 1, 1, 1), "fwd_auto_kernel<4, 7, 2, 2, 4, 14>"),
]


@pytest.mark.parametrize("g,kernel", COMBINED, ids=[k for _, k in COMBINED])
def test_fwd_auto_single_main_kernel(g, kernel):
    """st_conv_fwd_auto where one main kernel holds both forms: it is the instance expected for the
    geometry, and with few / many zeros the result is bit-identical to the dense / zero-skipping entry
    point's and agrees with the oracle (sampled outputs: the tensors have up to 50 M elements)."""
    assert st.st_conv_kernel_name(desc_of(g), st.ST_PASS_FWD_AUTO) == kernel
    for p, form in ((0.1, True), (0.7, False)):
        x, w, _ = synth(g, p, p, seed=65)
        L = DeviceLayer(g, x, w, None)
        got = L.fwd("auto", raw=True)
        assert torch.equal(got, L.fwd(form, raw=True)), f"p={p}: not the form {form!r}"
        assert not torch.equal(got, L.fwd(not form, raw=True)), "forms indistinguishable: test is void"
        cy = sample_coords(g.y_shape, 2048, 7)
        ref, ref_abs = st_ref.conv_fwd_at(g, x, w, cy)
        assert_close(gather_activations(got, cy), ref, ref_abs, f"{kernel} p={p}")


def test_bwi_auto_single_main_kernel():
    """The same for st_conv_bwi_auto (the kernel runs on dy with the filters transposed)."""
    g = Geom(8, 128, 64, 56, 56, 3, 3, 1, 1, 1, 1)
    assert st.st_conv_kernel_name(desc_of(g), st.ST_PASS_BWI_AUTO) == "fwd_auto_kernel<4, 7, 2, 4, 4, 8>"
    for p, form in ((0.1, True), (0.7, False)):
        x, w, dy = synth(g, p, p, seed=66)
        L = DeviceLayer(g, None, w, dy)
        got = L.bwi("auto", raw=True)
        assert torch.equal(got, L.bwi(form, raw=True)), f"p={p}: not the form {form!r}"
        cx = sample_coords(g.x_shape, 2048, 8)
        ref, ref_abs = st_ref.conv_bwi_at(g, dy, w, cx)
        assert_close(gather_activations(got, cx), ref, ref_abs, f"BWI auto p={p}")


def test_fwd_bwi_auto_small_launch():
    """A launch of few tasks (both forms split their reduction over wavefronts / workgroups): the
    usual break-even applies, and both forms agree with the oracle."""
    g = Geom(1, 256, 256, 7, 7, 3, 3, 1, 1, 1, 1)
    assert st.st_conv_sparse_threshold(desc_of(g), st.ST_PASS_FWD) == 250
    for p, form in ((0.1, True), (0.9, False)):
        x, w, dy = synth(g, p, p, seed=63)
        L = DeviceLayer(g, x, w, dy)
        assert not np.array_equal(L.fwd(False), L.fwd(True)), "forms indistinguishable: test is void"
        assert np.array_equal(L.fwd("auto"), L.fwd(form))
        assert np.array_equal(L.bwi("auto"), L.bwi(form))
        check_all_passes_full(g, x, w, dy, f"small launch p={p}", passes=("fwd", "bwi"))


def test_fwd_auto_1x1_never_takes_the_narrow_sparse_form():
    g = Geom(2, 64, 64, 12, 12, 1, 1)
    x, w, dy = synth(g, 0.95, 0.95, seed=62)
    L = DeviceLayer(g, x, w, dy)
    assert np.array_equal(L.fwd("auto"), L.fwd(True))
    assert np.array_equal(L.bwi("auto"), L.bwi(True))


def test_dead_channels_are_skipped_correctly():
    """Whole channels of an image that are zero (no filter load, no mask pass in FWD/BWI): every
    count of alive channels per 16-channel block, a dead first channel, dead blocks, dead images."""
    g = Geom(3, 80, 128, 12, 16, 3, 3, 1, 1, 1, 1)
    x, w, dy = synth(g, 0.3, 0.3, seed=71)
    # image 0: block b keeps its first b*3 + 1 channels' complement pattern; image 1: random; image 2: all dead
    for b in range(5):
        alive = {0: [], 1: [0], 2: [15], 3: [1, 2, 3], 4: list(range(1, 16))}[b]
        for ci in range(16):
            if ci not in alive:
                x[0, b * 16 + ci] = 0.0
    x[1:2] = stgen.dead_channels(x[1:2], 0.5, 72)
    x[2] = 0.0
    dy[0, 5:] = 0.0                                        # BWI: K = 128, most channels of image 0 dead
    dy[1:2] = stgen.dead_channels(dy[1:2], 0.6, 73)
    dy[2, ::2] = -0.0                                      # -0 planes count as dead
    check_all_passes_full(g, x, w, dy, "dead-channels")
    # 1x1 and stride 2 run the same channel loop
    for g2 in (Geom(2, 64, 256, 9, 9, 1, 1), Geom(2, 48, 128, 14, 14, 3, 3, 2, 2, 1, 1)):
        x, w, dy = synth(g2, 0.3, 0.3, seed=74)
        x = stgen.dead_channels(x, 0.6, 75)
        dy = stgen.dead_channels(dy, 0.6, 76)
        check_all_passes_full(g2, x, w, dy, "dead-channels-2")
    # BWW hands the channels that have a non-zero in the first tile of a workgroup's range to its wavefronts first
    # (a prediction of the dead planes): channels that are zero in that tile and alive elsewhere, alive in that
    # tile only, a partly filled group of 64 channels, and the same with dy as the tested operand
    g3 = Geom(2, 144, 80, 20, 24, 3, 3, 1, 1, 1, 1)
    x, w, dy = synth(g3, 0.3, 0.3, seed=77)
    x = stgen.dead_channels(x, 0.7, 78)
    dy = stgen.dead_channels(dy, 0.5, 79)
    x[:, ::5, :8, :8] = 0.0
    x[:, 3::7, 8:, :] = 0.0
    x[:, 3::7, :, 8:] = 0.0
    check_all_passes_full(g3, x, w, dy, "dead-channels-bww")


def random_geometries(count, seed):
    """Seeded mix of small geometries over everything the descriptor allows: filter sizes 1/3/5
    (square and not), strides 1/2, paddings 0..2, odd image sizes, channel counts 16..160."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        R, S = (int(v) for v in rng.choice([1, 3, 3, 3, 5], 2))
        if rng.random() < 0.7:
            S = R
        sw = sh = int(rng.choice([1, 1, 2]))
        pw, ph = int(rng.integers(0, 3)), int(rng.integers(0, 3))
        if rng.random() < 0.6:
            pw, ph = (R - 1) // 2, (S - 1) // 2
        H, W = int(rng.integers(3, 21)), int(rng.integers(3, 21))
        if H + 2 * ph < S or W + 2 * pw < R:
            continue
        C, K = 16 * int(rng.integers(1, 11)), 16 * int(rng.integers(1, 11))
        out.append(Geom(int(rng.integers(1, 4)), C, K, H, W, R, S, sw, sh, pw, ph))
    return out


RANDOM_GEOMS = random_geometries(120, seed=2024)


@pytest.mark.parametrize("i", range(len(RANDOM_GEOMS)))
def test_random_geometries_all_entry_points(i):
    g = RANDOM_GEOMS[i]
    px, pdy = [(0.5, 0.5), (0.2, 0.8), (0.9, 0.3)][i % 3]
    x, w, dy = synth(g, px, pdy, seed=100 + i)
    if i % 4 == 0:
        x = stgen.dead_channels(x, 0.4, 900 + i)
    check_all_passes_full(g, x, w, dy, f"random#{i} {g}")


def wide_geometries(count, seed):
    """Seeded geometries of the tiled paths with up to 640 channels and up to 30 x 30 pixels: every
    channel split, several 64-channel groups, ragged tiles."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        R = int(rng.choice([1, 3, 3]))
        s = int(rng.choice([1, 1, 1, 2])) if R == 3 else 1
        H, W = int(rng.integers(5, 31)), int(rng.integers(5, 31))
        C, K = 16 * int(rng.integers(1, 41)), 16 * int(rng.integers(1, 41))
        if C * K * R * R * H * W * 2 > 4e9:
            continue
        out.append(Geom(int(rng.integers(1, 4)), C, K, H, W, R, R, s, s, (R - 1) // 2, (R - 1) // 2))
    return out


WIDE_GEOMS = wide_geometries(40, seed=6)


@pytest.mark.parametrize("i", range(len(WIDE_GEOMS)))
def test_wide_geometries_all_entry_points(i):
    g = WIDE_GEOMS[i]
    px, pdy = [(0.5, 0.6), (0.8, 0.2), (0.3, 0.3)][i % 3]
    x, w, dy = synth(g, px, pdy, seed=5000 + i)
    check_all_passes_full(g, x, w, dy, f"wide#{i} {g}")


def test_config3_resnet3_2_full():
    """N=32, C=K=128, 28x28, 3x3: x 50 % zeros, dy 45 % zeros; every element checked."""
    L = stgen.RESNET3_2
    g = geom_of(L)
    x, w, dy = stgen.make_layer_tensors(L, seed=0)
    check_all_passes_full(g, x, w, dy, "config3")


def test_config2_vgg3_2_full():
    """The vgg3_2-shaped workload at full size (N=16, 256->256 @56x56, x 60 % / dy 50 % zeros): every
    element of y, dx and dw of every entry point against the oracle."""
    L = stgen.VGG3_2_N16
    g = geom_of(L)
    x, w, dy = stgen.make_layer_tensors(L, seed=0)
    assert abs(stgen.zero_fraction(x) - 0.6) < 0.002 and abs(stgen.zero_fraction(dy) - 0.5) < 0.002
    check_all_passes_full(g, x, w, dy, "config2")


@pytest.mark.parametrize("layer", stgen.BOTTLENECK, ids=[l.name for l in stgen.BOTTLENECK])
def test_config4_bottleneck_full(layer):
    """The three layers of the ResNet-50 bottleneck at N=32, every element of every output."""
    g = geom_of(layer)
    x, w, dy = stgen.make_layer_tensors(layer, seed=0)
    check_all_passes_full(g, x, w, dy, "config4-" + layer.name)


VGG_SMALL = [l for l in stgen.vgg16_stack(0.5) if l.H <= 28]


@pytest.mark.parametrize("layer", [l for l in VGG_SMALL if l.H == 14][:1] + [l for l in VGG_SMALL if l.H == 28][:2],
                         ids=lambda l: l.name)
def test_config5_vgg_late_layers(layer):
    g = geom_of(layer)
    x, w, dy = stgen.make_layer_tensors(layer, seed=1)
    if layer.H == 14:
        check_all_passes_full(g, x, w, dy, "config5-" + layer.name)
    else:
        check_all_passes_sampled(g, x, w, dy, "config5-" + layer.name, n_samples=2048, n_bww=256)


def test_config5_vgg1_2_full_size_sampled():
    """The largest layer of the VGG16 stack (N=32, 64->64 @224x224, 411 MB per activation tensor):
    exercises the 64-channel tile configuration, 25088 tiles per pass and 64-bit offsets."""
    layer = stgen.vgg16_stack(0.5)[0]
    assert layer.name == "vgg1_2" and layer.N == 32
    g = geom_of(layer)
    x, w, dy = stgen.make_layer_tensors(layer, seed=3)
    check_all_passes_sampled(g, x, w, dy, "config5-vgg1_2", n_samples=4096, n_bww=128)


@pytest.mark.parametrize("name,p", [("vgg2_1", 0.3), ("vgg2_2", 0.7), ("vgg3_1", 0.5), ("vgg3_2", 0.9),
                                    ("vgg4_3", 0.0), ("vgg5_2", 0.7)])
def test_config5_vgg_layers_full_batch_sampled(name, p):
    """The other VGG16 layer shapes at the full minibatch N=32, one swept zero fraction each."""
    layer = [l for l in stgen.vgg16_stack(p) if l.name == name][0]
    g = geom_of(layer)
    x, w, dy = stgen.make_layer_tensors(layer, seed=4)
    check_all_passes_sampled(g, x, w, dy, f"config5-{name}-p{p}", n_samples=2048, n_bww=128)


TABLE1_REST = [l for l in stgen.table1_layers(32, 0.5, 0.6) if l.name.startswith("resnet") and
               l.name not in ("resnet2_1b", "resnet2_2", "resnet2_3", "resnet3_2")]


@pytest.mark.parametrize("layer", TABLE1_REST, ids=[l.name for l in TABLE1_REST])
def test_table1_resnet_layers_full_batch_sampled(layer):
    """The ResNet rows of Table 1 not covered above (the stride-2 layers and the late 1x1 layers
    included) at N=32, all entry points, on sampled outputs."""
    g = geom_of(layer)
    x, w, dy = stgen.make_layer_tensors(layer, seed=6)
    check_all_passes_sampled(g, x, w, dy, f"table1-{layer.name}", n_samples=2048, n_bww=128)


def test_side_stream_and_reused_workspace():
    """Calls on a non-default stream with one workspace reused by consecutive calls give the same
    bits as calls on the default stream (the library only enqueues; it never synchronises)."""
    g = Geom(2, 64, 128, 16, 16, 3, 3, 1, 1, 1, 1)
    x, w, dy = synth(g, 0.5, 0.5, seed=11)
    L = DeviceLayer(g, x, w, dy)
    ref_y, ref_dx, ref_dw = L.fwd(False), L.bwi(False), L.bww(False)
    d = L.d
    need = max(st.st_conv_workspace_bytes(d, p, dn) for p in (0, 1, 2) for dn in (False, True))
    side = torch.cuda.Stream()
    ws = torch.empty(need // 4 + 64, dtype=torch.float32, device="cuda")
    y = torch.empty((g.N, g.K // 16, g.OH, g.OW, 16), device="cuda")
    dx = torch.empty((g.N, g.C // 16, g.H, g.W, 16), device="cuda")
    dw = torch.empty((g.K // 16, g.C // 16, g.S, g.R, 16, 16), device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for _ in range(2):
            st.st_conv_fwd(d, L.x, L.w, y, ws, side)
            st.st_conv_bwi(d, L.dy, L.w, dx, ws, side)
            st.st_conv_bww(d, L.x, L.dy, dw, ws, side)
            st.st_conv_fwd_dense(d, L.x, L.w, y, ws, side)
            st.st_conv_fwd(d, L.x, L.w, y, ws, side)
    side.synchronize()
    assert np.array_equal(st.unpack_activations(y.cpu().numpy()), ref_y)
    assert np.array_equal(st.unpack_activations(dx.cpu().numpy()), ref_dx)
    assert np.array_equal(st.unpack_filters(dw.cpu().numpy()), ref_dw)


@pytest.mark.parametrize("p", [0.0, 0.3, 0.7, 0.9])
def test_config5_sweep_levels_on_vgg5(p):
    layer = stgen.vgg16_stack(p, n=8)[-1]
    g = geom_of(layer)
    x, w, dy = stgen.make_layer_tensors(layer, seed=2)
    check_all_passes_sampled(g, x, w, dy, f"vgg5_3 p={p}", n_samples=2048, n_bww=256)


# One layer of each tile configuration of the 3x3 kernels (64 produced channels: 8x8 tiles, one channel
# per lane, in FWD and BWI of vgg1_2 and in BWI of vgg2_1; multiples of 128: 4x8 tiles, two per lane;
# rows of 28 and 14 pixels: 7-wide tiles) at the full minibatch and at every swept zero fraction.
SWEEP_LAYERS = ("vgg1_2", "vgg2_1", "vgg3_2", "vgg4_2", "vgg5_1")


@pytest.mark.parametrize("name", SWEEP_LAYERS)
def test_config5_all_sweep_levels_full_batch_sampled(name):
    """N=32, zero fraction of x and of dy swept over {0, 30, 50, 70, 90} %: the tensors of one stream
    at several fractions share their normals and uniforms, which are drawn once."""
    layer = [l for l in stgen.vgg16_stack(0.5) if l.name == name][0]
    g = geom_of(layer)
    seed = 40 + SWEEP_LAYERS.index(name)
    z = stgen.normal(4 * seed, int(np.prod(g.x_shape)))
    w = stgen.he_normal(g.w_shape, 4 * seed + 1)
    gn = stgen.normal(4 * seed + 2, int(np.prod(g.y_shape)))
    u = stgen.uniform(4 * seed + 3, int(np.prod(g.y_shape)))
    for p in (0.0, 0.3, 0.5, 0.7, 0.9):
        x = stgen.relu_from_normal(z, p).reshape(g.x_shape)
        dy = stgen.mask_from_uniform(gn, u, p).reshape(g.y_shape)
        assert abs(stgen.zero_fraction(x) - p) < 0.002 and abs(stgen.zero_fraction(dy) - p) < 0.002
        check_all_passes_sampled(g, x, w, dy, f"config5-{name}-p{p}", n_samples=1024, n_bww=64, seed=int(100 * p))
