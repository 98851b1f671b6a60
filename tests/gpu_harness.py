"""Helpers for the GPU parity tests: upload plain host tensors in the library's blocked layout,
call the C ABI through the Python binding, download, and compare with the CPU oracle.

Bar (stated by the benchmark definition): max |gpu - ref| / sum|terms| <= 1e-4 per element, and
an element whose terms are all zero must come back as exactly +-0.
"""
import numpy as np
import torch

import paper_1911_10175_amd as st
from oracle import st_ref
from oracle.st_ref import Geom

TOL = 1e-4


def desc_of(g: Geom) -> st.ConvDesc:
    return st.ConvDesc(g.N, g.C, g.K, g.H, g.W, g.R, g.S, g.stride_w, g.stride_h, g.pad_w, g.pad_h)


def dev(a_packed: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(a_packed).to("cuda")


def nan_like(shape) -> torch.Tensor:
    return torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")


def workspace(d: st.ConvDesc, conv_pass: int, dense: bool):
    need = st.st_conv_workspace_bytes(d, conv_pass, dense)
    if need == 0:
        return None
    return torch.empty((need + 3) // 4, dtype=torch.float32, device="cuda")


class DeviceLayer:
    """Device copies (blocked layout) of one layer's tensors."""

    def __init__(self, g: Geom, x=None, w=None, dy=None):
        self.g = g
        self.d = desc_of(g)
        self.x = dev(st.pack_activations(x)) if x is not None else None
        self.w = dev(st.pack_filters(w)) if w is not None else None
        self.dy = dev(st.pack_activations(dy)) if dy is not None else None

    def fwd(self, dense=False, raw=False):
        """dense = False: st_conv_fwd; True: st_conv_fwd_dense; "auto": st_conv_fwd_auto.
        raw = True returns the device tensor in the blocked layout instead of a plain host array."""
        g = self.g
        y = nan_like((g.N, g.K // 16, g.OH, g.OW, 16))
        if dense == "auto":
            ws = self.auto_ws = workspace(self.d, st.ST_PASS_FWD_AUTO, False)
            st.st_conv_fwd_auto(self.d, self.x, self.w, y, ws)
        else:
            ws = workspace(self.d, st.ST_PASS_FWD, dense)
            (st.st_conv_fwd_dense if dense else st.st_conv_fwd)(self.d, self.x, self.w, y, ws)
        torch.cuda.synchronize()
        return y if raw else st.unpack_activations(y.cpu().numpy())

    def bwi(self, dense=False, raw=False):
        g = self.g
        dx = nan_like((g.N, g.C // 16, g.H, g.W, 16))
        if dense == "auto":
            ws = self.auto_ws = workspace(self.d, st.ST_PASS_BWI_AUTO, False)
            st.st_conv_bwi_auto(self.d, self.dy, self.w, dx, ws)
        else:
            ws = workspace(self.d, st.ST_PASS_BWI, dense)
            (st.st_conv_bwi_dense if dense else st.st_conv_bwi)(self.d, self.dy, self.w, dx, ws)
        torch.cuda.synchronize()
        return dx if raw else st.unpack_activations(dx.cpu().numpy())

    def bww(self, dense=False, raw=False):
        """dense = False: st_conv_bww (tests x); True: st_conv_bww_dense; "dy": st_conv_bww_dy;
        "auto": st_conv_bww_auto (its workspace is kept in self.auto_ws for inspection)."""
        g = self.g
        dw = nan_like((g.K // 16, g.C // 16, g.S, g.R, 16, 16))
        if dense == "dy":
            ws = workspace(self.d, st.ST_PASS_BWW_DY, False)
            st.st_conv_bww_dy(self.d, self.x, self.dy, dw, ws)
        elif dense == "auto":
            ws = self.auto_ws = workspace(self.d, st.ST_PASS_BWW_AUTO, False)
            st.st_conv_bww_auto(self.d, self.x, self.dy, dw, ws)
        else:
            ws = workspace(self.d, st.ST_PASS_BWW, dense)
            (st.st_conv_bww_dense if dense else st.st_conv_bww)(self.d, self.x, self.dy, dw, ws)
        torch.cuda.synchronize()
        return dw if raw else st.unpack_filters(dw.cpu().numpy())


def bww_variants(variants):
    """The BWW entry points to check: the dy-testing and the self-selecting one ride along with the
    x-testing one."""
    return tuple(variants) + (("dy", "auto") if False in variants else ())


def fwd_variants(variants):
    """FWD / BWI entry points to check: the self-selecting one rides along when both forms are checked."""
    return tuple(variants) + (("auto",) if False in variants and True in variants else ())


def assert_close(got, ref, ref_abs, what):
    assert got.shape == ref.shape, what
    assert np.isfinite(got).all(), f"{what}: non-finite or unwritten output elements"
    err, bad_zero = st_ref.rel_err(got, ref, ref_abs)
    assert bad_zero == 0, f"{what}: {bad_zero} elements with all-zero terms are not zero"
    assert err <= TOL, f"{what}: max relative error {err:.3e} > {TOL}"
    return err


def check_all_passes_full(g: Geom, x, w, dy, label, passes=("fwd", "bwi", "bww"), variants=(False, True)):
    """Element-by-element parity of the sparse (dense=False) and dense entry points."""
    L = DeviceLayer(g, x, w, dy)
    errs = {}
    if "fwd" in passes:
        ref, ref_abs = st_ref.conv_fwd(g, x, w)
        for dense in fwd_variants(variants):
            errs["fwd", dense] = assert_close(L.fwd(dense), ref, ref_abs, f"{label} FWD dense={dense}")
    if "bwi" in passes:
        ref, ref_abs = st_ref.conv_bwi(g, dy, w)
        for dense in fwd_variants(variants):
            errs["bwi", dense] = assert_close(L.bwi(dense), ref, ref_abs, f"{label} BWI dense={dense}")
    if "bww" in passes:
        ref, ref_abs = st_ref.conv_bww(g, x, dy)
        for dense in bww_variants(variants):
            errs["bww", dense] = assert_close(L.bww(dense), ref, ref_abs, f"{label} BWW dense={dense}")
    return errs


def sample_coords(shape, n, seed):
    rng = np.random.default_rng(seed)
    cols = [rng.integers(0, s, n) for s in shape]
    c = np.stack(cols, axis=1).astype(np.int32)
    # always include the corners of the index space (image borders, first/last channel)
    corners = np.array([[0] * len(shape), [s - 1 for s in shape]], dtype=np.int32)
    return np.concatenate([corners, c], axis=0)


def gather_activations(t: torch.Tensor, coords: np.ndarray) -> np.ndarray:
    """Elements (n, c, h, w) of a device tensor in the blocked layout [N][C/16][H][W][16]; every
    element of the tensor must be finite (checked on the device)."""
    assert bool(torch.isfinite(t).all()), "non-finite or unwritten output elements"
    c = torch.from_numpy(coords.astype(np.int64)).to(t.device)
    return t[c[:, 0], c[:, 1] // 16, c[:, 2], c[:, 3], c[:, 1] % 16].cpu().numpy()


def gather_filters(t: torch.Tensor, coords: np.ndarray) -> np.ndarray:
    """Elements (k, c, v, u) of a device tensor in the blocked layout [K/16][C/16][S][R][16 c][16 k]."""
    assert bool(torch.isfinite(t).all()), "non-finite or unwritten output elements"
    c = torch.from_numpy(coords.astype(np.int64)).to(t.device)
    return t[c[:, 0] // 16, c[:, 1] // 16, c[:, 2], c[:, 3], c[:, 1] % 16, c[:, 0] % 16].cpu().numpy()


def check_all_passes_sampled(g: Geom, x, w, dy, label, n_samples=4096, seed=0, variants=(False, True),
                             n_bww=512):
    """Parity on seeded sampled outputs, each computed one by one by the oracle; for tensors too
    large for a full oracle pass.  The samples are gathered on the device (the whole output is only
    checked for non-finite values there), so a 411 MB output costs no download."""
    L = DeviceLayer(g, x, w, dy)
    cy = sample_coords(g.y_shape, n_samples, seed)
    ref, ref_abs = st_ref.conv_fwd_at(g, x, w, cy)
    for dense in fwd_variants(variants):
        assert_close(gather_activations(L.fwd(dense, raw=True), cy), ref, ref_abs, f"{label} FWD dense={dense} (sampled)")
    cx = sample_coords(g.x_shape, n_samples, seed + 1)
    ref, ref_abs = st_ref.conv_bwi_at(g, dy, w, cx)
    for dense in fwd_variants(variants):
        assert_close(gather_activations(L.bwi(dense, raw=True), cx), ref, ref_abs, f"{label} BWI dense={dense} (sampled)")
    cw = sample_coords(g.w_shape, n_bww, seed + 2)
    ref, ref_abs = st_ref.conv_bww_at(g, x, dy, cw)
    for dense in bww_variants(variants):
        assert_close(gather_filters(L.bww(dense, raw=True), cw), ref, ref_abs, f"{label} BWW dense={dense} (sampled)")
