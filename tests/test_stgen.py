"""Checks of the seeded input generators (no convolution arithmetic involved)."""
import numpy as np
import pytest

import stgen


def test_reproducible_and_stream_separated():
    a = stgen.normal(7, 1000)
    b = stgen.normal(7, 1000)
    c = stgen.normal(8, 1000)
    np.testing.assert_array_equal(a, b)
    assert not np.array_equal(a, c)
    # counter based: a prefix of a longer draw equals the shorter draw
    np.testing.assert_array_equal(stgen.normal(7, 5_000_000)[:1000], a)


def test_normal_moments():
    z = stgen.normal(3, 2_000_000)
    assert abs(z.mean()) < 4 / np.sqrt(z.size)
    assert abs(z.var() - 1.0) < 0.005
    assert abs(np.mean(z ** 3)) < 0.01
    assert abs(np.mean(z ** 4) - 3.0) < 0.03
    u = stgen.uniform(3, 1_000_000)
    assert 0.0 <= u.min() and u.max() < 1.0 and abs(u.mean() - 0.5) < 0.002


@pytest.mark.parametrize("p", [0.3, 0.4, 0.45, 0.5, 0.55, 0.6, 0.7, 0.9])
def test_relu_sparse_hits_target_fraction(p):
    n = 1_000_000
    x = stgen.relu_sparse((n,), p, 11)
    assert x.dtype == np.float32 and (x >= 0).all()
    sigma = np.sqrt(p * (1 - p) / n)
    assert abs(stgen.zero_fraction(x) - p) < 4 * sigma
    assert not np.signbit(x[x == 0]).any()          # ReLU zeros are +0


def test_centered_relu_gives_half_zeros():
    """Sec. 2.2: ReLU of a zero-centred distribution is 50 % sparse (threshold t = 0)."""
    assert stgen.relu_threshold(0.5) == 0.0
    assert abs(stgen.relu_threshold(0.6) - 0.2533) < 1e-4
    assert abs(stgen.relu_threshold(0.9) - 1.2816) < 1e-4


def test_dense_when_p_is_zero():
    x = stgen.relu_sparse((100000,), 0.0, 5)
    assert stgen.zero_fraction(x) == 0.0 and (x < 0).any()


@pytest.mark.parametrize("q", [0.3, 0.45, 0.5, 0.9])
def test_bernoulli_masked(q):
    n = 1_000_000
    dy = stgen.bernoulli_masked((n,), q, 21, 22)
    sigma = np.sqrt(q * (1 - q) / n)
    assert abs(stgen.zero_fraction(dy) - q) < 4 * sigma
    zeros = dy[dy == 0]
    assert np.signbit(zeros).any() and (~np.signbit(zeros)).any()   # both +0 and -0 occur
    nz = dy[dy != 0]
    assert abs(nz.mean()) < 0.01 and abs(nz.var() - 1.0) < 0.01


def test_he_normal_variance():
    w = stgen.he_normal((256, 128, 3, 3), 9)
    assert w.shape == (256, 128, 3, 3) and w.dtype == np.float32
    assert abs(w.var() / (2.0 / (128 * 9)) - 1.0) < 0.01


def test_relu_grad_mask_is_strict():
    y = np.array([-1.0, 0.0, -0.0, 2.0, 1e-30], dtype=np.float32)
    d = stgen.relu_grad(y, 4)
    assert (d[:3] == 0).all() and d[3] != 0 and d[4] != 0


def test_workload_table():
    assert stgen.VGG3_2_N16.flops == 2 * 16 * 256 * 256 * 56 * 56 * 9
    stack = stgen.vgg16_stack(0.5)
    assert len(stack) == 12 and sum(l.flops for l in stack) == 976_635_297_792
    x, w, dy = stgen.make_layer_tensors(stgen.TINY, seed=0)
    assert x.shape == (1, 16, 8, 8) and w.shape == (16, 16, 3, 3) and dy is None


def test_dead_channels_zero_whole_planes():
    a = stgen.relu_sparse((4, 32, 5, 6), 0.0, 7)
    b = stgen.dead_channels(a, 0.5, 8)
    planes = np.abs(b).reshape(4 * 32, -1).sum(axis=1)
    dead = int((planes == 0).sum())
    assert 40 < dead < 90                                  # about half of the 128 planes
    alive = planes != 0
    assert np.array_equal(b.reshape(128, -1)[alive], a.reshape(128, -1)[alive])
    assert np.array_equal(stgen.dead_channels(a, 0.5, 8), b)      # deterministic
