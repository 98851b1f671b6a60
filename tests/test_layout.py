"""The blocked layouts of include/st_conv.h against their index formulas (SparseTrain Sec. 3.2.5:
channel tile lowest for activations; k vector, c tile, filter width for filters)."""
import numpy as np
import torch

from paper_1911_10175_amd import pack_activations, pack_filters, unpack_activations, unpack_filters


def test_activation_layout_formula():
    n, c, h, w = 2, 48, 3, 5
    a = np.arange(n * c * h * w, dtype=np.float32).reshape(n, c, h, w)
    flat = pack_activations(a).ravel()
    for (i, ch, y, x) in [(0, 0, 0, 0), (1, 47, 2, 4), (1, 17, 1, 3), (0, 31, 2, 0)]:
        off = ((((i * (c // 16) + ch // 16) * h + y) * w + x) * 16) + ch % 16
        assert flat[off] == a[i, ch, y, x]
    assert (unpack_activations(pack_activations(a)) == a).all()
    t = torch.from_numpy(a)
    assert torch.equal(pack_activations(t), torch.from_numpy(pack_activations(a)))
    assert torch.equal(unpack_activations(pack_activations(t)), t)


def test_filter_layout_formula():
    k, c, s, r = 32, 48, 2, 3
    f = np.arange(k * c * s * r, dtype=np.float32).reshape(k, c, s, r)
    flat = pack_filters(f).ravel()
    for (kk, cc, v, u) in [(0, 0, 0, 0), (31, 47, 1, 2), (17, 5, 0, 1), (3, 33, 1, 0)]:
        off = (((((kk // 16) * (c // 16) + cc // 16) * s + v) * r + u) * 16 + cc % 16) * 16 + kk % 16
        assert flat[off] == f[kk, cc, v, u]
    assert (unpack_filters(pack_filters(f)) == f).all()
    t = torch.from_numpy(f)
    assert torch.equal(pack_filters(t), torch.from_numpy(pack_filters(f)))
    assert torch.equal(unpack_filters(pack_filters(t)), t)


def test_harness_gathers_index_the_blocked_layouts():
    """The GPU tests pick sampled outputs straight out of blocked device tensors: the index arithmetic
    they use must agree with unpacking the whole tensor (run here on CPU tensors)."""
    from tests.gpu_harness import gather_activations, gather_filters, sample_coords
    a = np.random.default_rng(0).standard_normal((2, 48, 5, 7)).astype(np.float32)
    ca = sample_coords(a.shape, 200, 1)
    assert (gather_activations(torch.from_numpy(pack_activations(a)), ca) == a[tuple(ca.T)]).all()
    f = np.random.default_rng(1).standard_normal((32, 48, 3, 2)).astype(np.float32)
    cf = sample_coords(f.shape, 200, 2)
    assert (gather_filters(torch.from_numpy(pack_filters(f)), cf) == f[tuple(cf.T)]).all()
