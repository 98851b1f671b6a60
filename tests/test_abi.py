"""Host-side checks of the C ABI: the library loads without a GPU, exports every symbol the
public header declares, and validates arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_1911_10175_amd as st
from paper_1911_10175_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "st_conv.h")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(st_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    lib = st.load_library()
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings_and_version():
    assert st.st_status_str(0) == "ok"
    seen = {st.st_status_str(i) for i in range(7)}
    assert len(seen) == 7 and all(seen)
    assert st.st_status_str(99) == "unknown status"
    assert re.fullmatch(r"\d+\.\d+", st.st_conv_version())


def test_validation_happens_on_the_host():
    good = st.ConvDesc(1, 16, 16, 8, 8, 3, 3, 1, 1, 1, 1)
    lib = st.load_library()
    # NULL descriptor
    assert lib.st_conv_fwd(None, None, None, None, None, 0, None) == 1
    # NULL tensors
    assert st.st_conv_fwd(good, None, None, None, check=False) == 1
    assert st.st_conv_bwi_dense(good, None, None, None, check=False) == 1
    assert st.st_conv_bww(good, None, None, None, check=False) == 1
    assert st.st_conv_bww_dy(good, None, None, None, check=False) == 1
    assert st.st_conv_bww_auto(good, None, None, None, check=False) == 1
    assert st.st_conv_fwd_auto(good, None, None, None, check=False) == 1
    assert st.st_conv_bwi_auto(good, None, None, None, check=False) == 1
    bad = [st.ConvDesc(0, 16, 16, 8, 8, 3, 3), st.ConvDesc(1, 8, 16, 8, 8, 3, 3, 1, 1, 1, 1),
           st.ConvDesc(1, 16, 24, 8, 8, 3, 3, 1, 1, 1, 1), st.ConvDesc(1, 16, 16, 2, 8, 3, 3),
           st.ConvDesc(1, 16, 16, 8, 8, 3, 3, 0, 1), st.ConvDesc(1, 16, 16, 8, 8, 3, 3, 1, 1, -1, 0)]
    for d in bad:
        for fn in (st.st_conv_fwd, st.st_conv_fwd_dense, st.st_conv_bwi, st.st_conv_bwi_dense,
                   st.st_conv_bww, st.st_conv_bww_dense, st.st_conv_bww_dy, st.st_conv_bww_auto,
                   st.st_conv_fwd_auto, st.st_conv_bwi_auto):
            assert fn(d, 256, 256, 256, check=False) == 2, d
        assert st.st_conv_workspace_bytes(d, st.ST_PASS_BWI) == 0
    with pytest.raises(st.StConvError) as e:
        st.st_conv_fwd(bad[0], 256, 256, 256)
    assert e.value.status == 2


def test_misaligned_tensors_and_oversized_images_are_refused_on_the_host():
    """The kernels use 16-byte vector accesses and keep offsets within one image's channel block in
    int: both limits are statuses, never faults."""
    d = st.ConvDesc(1, 16, 16, 8, 8, 3, 3, 1, 1, 1, 1)
    fns = (st.st_conv_fwd, st.st_conv_fwd_dense, st.st_conv_bwi, st.st_conv_bwi_dense, st.st_conv_bww,
           st.st_conv_bww_dense, st.st_conv_bww_dy, st.st_conv_bww_auto, st.st_conv_fwd_auto, st.st_conv_bwi_auto)
    for fn in fns:
        for args in ((256 + 4, 256, 256), (256, 256 + 16, 256), (256, 256, 256 + 32)):
            assert fn(d, *args, ws=4096, ws_bytes=1 << 30, check=False) == 6, fn
        assert fn(d, 256, None, 256 + 4, check=False) == 1          # NULL is reported before alignment
    assert "aligned" in st.st_status_str(6)
    # 2^27 pixels per image: (h*W + w) * 16 no longer fits an int
    big = st.ConvDesc(1, 16, 16, 1 << 14, 1 << 13, 1, 1)
    ok = st.ConvDesc(1, 16, 16, (1 << 14) - 1, 1 << 13, 1, 1)
    for fn in fns:
        assert fn(big, 256, 256, 256, ws=4096, ws_bytes=1 << 40, check=False) == 3, fn
    assert st.st_conv_workspace_bytes(big, st.ST_PASS_BWW) == 0
    assert st.st_conv_sparse_threshold(ok, st.ST_PASS_FWD) >= 0 and st.st_conv_sparse_threshold(big, st.ST_PASS_FWD) == -1


def test_library_reads_no_environment_variables():
    """Kernel shapes, reduction splits and workspace sizes depend on the descriptor alone."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--undefined-only", st.lib_path()], capture_output=True, text=True, check=True).stdout
    assert "getenv" not in out


def test_workspace_query_and_rejection():
    d = st.ConvDesc(16, 256, 256, 56, 56, 3, 3, 1, 1, 1, 1)
    # the tiled zero-skipping FWD / BWI read a copy of the filters in wavefront order: the produced
    # channels (K for FWD, C for BWI) rounded up to whole groups of 64
    assert st.st_conv_workspace_bytes(d, st.ST_PASS_FWD) == 256 * 256 * 9 * 4
    odd = st.ConvDesc(2, 48, 80, 12, 12, 3, 3, 1, 1, 1, 1)
    assert st.st_conv_workspace_bytes(odd, st.ST_PASS_FWD) == 128 * 48 * 9 * 4
    assert st.st_conv_workspace_bytes(odd, st.ST_PASS_BWI) == 64 * 80 * 9 * 4
    assert st.st_conv_fwd(d, 256, 256, 256, ws=None, check=False) == 4
    assert st.st_conv_fwd(d, 256, 256, 256, ws=4096 + 64, ws_bytes=1 << 30, check=False) == 4
    for dense in (False, True):
        need = st.st_conv_workspace_bytes(d, st.ST_PASS_BWI, dense)
        if need:
            fn = st.st_conv_bwi_dense if dense else st.st_conv_bwi
            # missing, too small and misaligned workspaces are refused before any launch
            assert fn(d, 256, 256, 256, ws=None, check=False) == 4
            assert fn(d, 256, 256, 256, ws=4096, ws_bytes=need - 1, check=False) == 4
            assert fn(d, 256, 256, 256, ws=4096 + 64, ws_bytes=need, check=False) == 4
        need = st.st_conv_workspace_bytes(d, st.ST_PASS_BWW, dense)
        if need:
            fn = st.st_conv_bww_dense if dense else st.st_conv_bww
            assert fn(d, 256, 256, 256, ws=None, check=False) == 4
            assert fn(d, 256, 256, 256, ws=4096, ws_bytes=need - 1, check=False) == 4
    # the dy-testing BWW always stages its partial sums, even a single one
    for dd in (d, st.ConvDesc(1, 512, 512, 8, 8, 3, 3, 1, 1, 1, 1)):
        need = st.st_conv_workspace_bytes(dd, st.ST_PASS_BWW_DY)
        assert need >= dd.K * dd.C * 9 * 4 and need % (dd.K * dd.C * 9 * 4) == 0
        assert st.st_conv_bww_dy(dd, 256, 256, 256, ws=None, check=False) == 4
        assert st.st_conv_bww_dy(dd, 256, 256, 256, ws=4096, ws_bytes=need - 1, check=False) == 4
        # the self-selecting form: counters plus the largest of the three forms it chooses from
        auto = st.st_conv_workspace_bytes(dd, st.ST_PASS_BWW_AUTO)
        assert auto == 256 + max(need, st.st_conv_workspace_bytes(dd, st.ST_PASS_BWW),
                                 st.st_conv_workspace_bytes(dd, st.ST_PASS_BWW, True))
        assert st.st_conv_bww_auto(dd, 256, 256, 256, ws=4096, ws_bytes=auto - 1, check=False) == 4
    # FWD / BWI with the form chosen on the device: counters + both forms' workspaces
    for pa, pb, fn in ((st.ST_PASS_FWD_AUTO, st.ST_PASS_FWD, st.st_conv_fwd_auto),
                       (st.ST_PASS_BWI_AUTO, st.ST_PASS_BWI, st.st_conv_bwi_auto)):
        need = st.st_conv_workspace_bytes(d, pa)
        assert need == 256 + st.st_conv_workspace_bytes(d, pb, False) + st.st_conv_workspace_bytes(d, pb, True)
        assert fn(d, 256, 256, 256, ws=None, check=False) == 4
        assert fn(d, 256, 256, 256, ws=4096, ws_bytes=need - 1, check=False) == 4
    # shapes served by the generic kernel need none
    assert st.st_conv_workspace_bytes(st.ConvDesc(1, 16, 16, 8, 8, 5, 5, 1, 1, 2, 2), st.ST_PASS_BWW_DY) == 0
    assert st.st_conv_workspace_bytes(st.ConvDesc(1, 16, 16, 8, 8, 5, 5, 1, 1, 2, 2), st.ST_PASS_FWD) == 0
    assert st.st_conv_workspace_bytes(d, 7) == 0


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_HERE", str(tmp_path))
    with pytest.raises(FileNotFoundError):
        binding.load_library()


def test_sparse_threshold_policy():
    """Break-even points of the self-selecting FWD / BWI entry points (host-side query)."""
    F, B = st.ST_PASS_FWD, st.ST_PASS_BWI
    vgg = st.ConvDesc(16, 256, 256, 56, 56, 3, 3, 1, 1, 1, 1)
    assert st.st_conv_sparse_threshold(vgg, F) == 250 and st.st_conv_sparse_threshold(vgg, B) == 250
    narrow = st.ConvDesc(16, 64, 64, 56, 56, 3, 3, 1, 1, 1, 1)
    assert st.st_conv_sparse_threshold(narrow, F) == 400
    # FWD vectorises over K, BWI over C
    mixed = st.ConvDesc(16, 64, 128, 56, 56, 3, 3, 1, 1, 1, 1)
    assert st.st_conv_sparse_threshold(mixed, F) == 250 and st.st_conv_sparse_threshold(mixed, B) == 400
    s2 = st.ConvDesc(8, 128, 128, 56, 56, 3, 3, 2, 2, 1, 1)
    assert st.st_conv_sparse_threshold(s2, F) == 800 and st.st_conv_sparse_threshold(s2, B) == 450
    pw = st.ConvDesc(8, 64, 256, 56, 56, 1, 1)
    assert st.st_conv_sparse_threshold(pw, F) == 1001 and st.st_conv_sparse_threshold(pw, B) == 1001
    # launches with few tasks split their reduction in both forms: same break-even as the large ones
    tiny = st.ConvDesc(32, 512, 512, 7, 7, 3, 3, 1, 1, 1, 1)
    assert st.st_conv_sparse_threshold(tiny, F) == 250 and st.st_conv_sparse_threshold(tiny, B) == 250
    # the dense form's workspace then also holds the partial outputs of its channel split
    assert st.st_conv_workspace_bytes(tiny, F, True) == 512 * 512 * 9 * 4 + 4 * 32 * 512 * 49 * 4      # 4 shares
    # only generic kernels: the test can only remove work
    assert st.st_conv_sparse_threshold(st.ConvDesc(1, 16, 16, 9, 9, 5, 5, 1, 1, 2, 2), F) == 0
    assert st.st_conv_sparse_threshold(st.ConvDesc(0, 16, 16, 9, 9, 3, 3), F) == -1
    assert st.st_conv_sparse_threshold(vgg, st.ST_PASS_BWW) == -1


def test_kernel_name_query():
    """Host-side: which instance of the zero-skipping FWD / BWI kernel a geometry gets."""
    vgg = st.ConvDesc(32, 256, 256, 56, 56, 3, 3, 1, 1, 1, 1)
    # rows of a multiple of 7 pixels: 7-wide tiles (five wavefronts per SIMD); otherwise 8-wide
    assert st.st_conv_kernel_name(vgg, st.ST_PASS_FWD) == "fwd_sparse_kernel<3, 3, 4, 7, 2, 4, 4, 1, 1, 0>"
    assert st.st_conv_kernel_name(st.ConvDesc(32, 256, 256, 64, 64, 3, 3, 1, 1, 1, 1), st.ST_PASS_FWD) == \
        "fwd_sparse_kernel<3, 3, 4, 8, 2, 4, 4, 1, 1, 0>"
    # 64 produced channels: one channel per lane on 8x8 tiles; FWD vectorises over K, BWI over C
    mixed = st.ConvDesc(32, 64, 128, 112, 112, 3, 3, 1, 1, 1, 1)
    assert st.st_conv_kernel_name(mixed, st.ST_PASS_FWD).startswith("fwd_sparse_kernel<3, 3, 4, 7, 2,")
    assert st.st_conv_kernel_name(mixed, st.ST_PASS_BWI).startswith("fwd_sparse_kernel<3, 3, 7, 7, 1,")      # sides of 7 n pixels: 7x7 tiles
    assert st.st_conv_kernel_name(st.ConvDesc(32, 128, 64, 64, 64, 3, 3, 1, 1, 1, 1), st.ST_PASS_FWD).startswith("fwd_sparse_kernel<3, 3, 8, 8, 1,")
    assert st.st_conv_kernel_name(st.ConvDesc(32, 512, 512, 28, 28, 3, 3, 1, 1, 1, 1), st.ST_PASS_FWD) == \
        "fwd_sparse_kernel<3, 3, 4, 7, 2, 4, 4, 1, 1, 0>"
    assert st.st_conv_kernel_name(st.ConvDesc(1, 16, 16, 9, 9, 5, 5, 1, 1, 2, 2), st.ST_PASS_FWD) is None   # generic kernel
    assert st.st_conv_kernel_name(vgg, st.ST_PASS_BWW) == "bww_sparse_kernel<3, 3, 7, 8, 0>"
    assert st.st_conv_kernel_name(st.ConvDesc(2, 64, 256, 56, 56, 1, 1), st.ST_PASS_BWW) == "pw_bww_sparse_kernel<4>"
    assert st.st_conv_kernel_name(vgg, st.ST_PASS_BWW_DY) is None
    lib = st.load_library()
    c = vgg._c()
    assert lib.st_conv_kernel_name(ctypes.byref(c), 0, None, 16) == 1
    small = ctypes.create_string_buffer(8)
    assert lib.st_conv_kernel_name(ctypes.byref(c), 0, small, 8) == 0 and small.value == b"fwd_spa"


def test_probe_arguments_are_checked_on_the_host():
    assert st.st_probe_issue_rate(0, 4, 10, None, check=False) == 1
    for bad in ((6, 4, 10), (-1, 4, 10), (0, 0, 10), (0, 4, 0), (0, (1 << 20) + 1, 1)):
        assert st.st_probe_issue_rate(*bad, 256, check=False) == 2
