"""st_conv_fwd_static (the entry point for callers that cannot allocate: its filter copy lives in an
array built into the library) against st_conv_fwd, through the C ABI: two calls in a row, the second
on a smaller layer, then the first again; results must be bit-identical to st_conv_fwd's (same
kernels) and within the benchmark's bar of the oracle."""
import numpy as np
import pytest
import torch

import stgen
from oracle import st_ref
from oracle.st_ref import Geom

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_1911_10175_amd as st
    from tests.gpu_harness import DeviceLayer, assert_close, nan_like


def run_static(L):
    g = L.g
    y = nan_like((g.N, g.K // 16, g.OH, g.OW, 16))
    st.st_conv_fwd_static(L.d, L.x, L.w, y)
    torch.cuda.synchronize()
    return y


def test_static_scratch_matches_workspace_entry_point_on_consecutive_calls():
    big = Geom(2, 128, 256, 20, 23, 3, 3, 1, 1, 1, 1)          # 1.2 MB filter copy, ragged tiles
    small = Geom(1, 48, 80, 9, 11, 3, 3, 1, 1, 1, 1)           # smaller copy: leaves stale data behind it
    pw = Geom(2, 64, 128, 12, 12, 1, 1)                        # 1x1 kernel family
    generic = Geom(1, 16, 32, 9, 9, 5, 5, 1, 1, 2, 2)          # no filter copy at all
    layers = []
    for i, g in enumerate((big, small, pw, generic)):
        x = stgen.relu_sparse(g.x_shape, 0.5, 900 + 4 * i)
        w = stgen.he_normal(g.w_shape, 901 + 4 * i)
        layers.append((g, x, w, DeviceLayer(g, x, w, None)))
    mem_before = torch.cuda.memory_allocated()
    for idx in (0, 1, 0, 2, 3, 1):
        g, x, w, L = layers[idx]
        want = L.fwd(False, raw=True)
        got = run_static(L)
        assert torch.equal(got, want), f"call on layer {idx}: differs from st_conv_fwd"
        ref, ref_abs = st_ref.conv_fwd(g, x, w)
        assert_close(st.unpack_activations(got.cpu().numpy()), ref, ref_abs, f"static FWD layer {idx}")
        del want, got
    assert torch.cuda.memory_allocated() == mem_before


def test_static_scratch_limit_and_argument_checks():
    # 1024 -> 1024 3x3: 37.7 MB of filter copy > 16 MiB, refused before any launch
    d = st.ConvDesc(1, 1024, 1024, 8, 8, 3, 3, 1, 1, 1, 1)
    assert st.st_conv_workspace_bytes(d, st.ST_PASS_FWD) > (16 << 20)
    assert st.st_conv_fwd_static(d, 256, 256, 256, check=False) == 4
    ok = st.ConvDesc(1, 512, 512, 8, 8, 3, 3, 1, 1, 1, 1)
    assert st.st_conv_workspace_bytes(ok, st.ST_PASS_FWD) <= (16 << 20)
    assert st.st_conv_fwd_static(ok, None, 256, 256, check=False) == 1
    assert st.st_conv_fwd_static(ok, 256, 256 + 4, 256, check=False) == 6
    assert st.st_conv_fwd_static(st.ConvDesc(0, 16, 16, 8, 8, 3, 3), 256, 256, 256, check=False) == 2
