"""Seeded synthetic tensors with the statistics of ReLU networks.

This module only draws numbers.  It holds none of the convolution arithmetic,
imports neither the CPU oracle nor the GPU package, and is the one piece both
sides of a parity test share: the same host arrays are handed to each.

The paper measured on synthetic tensors with random zero patterns at layer
shapes taken from VGG16 / ResNet (Sec. 4, Table 1) and notes that ReLU zeros
show no structure (Sec. 1); the generators below draw i.i.d. elements:

  relu_sparse      x  = max(0, z - t), z ~ N(0,1), t = Phi^-1(p)  -> fraction p of +0
  bernoulli_masked dy = g * m, g ~ N(0,1), m ~ Bernoulli(1-q)     -> fraction q of +-0
  he_normal        w  ~ N(0, 2 / (C*R*S))
  relu_grad        dy = g * (y > 0)  (ReLU' of Sec. 2.2 applied to a given y)

Random numbers come from a counter-based generator written here (a splitmix64
style mixer keyed by stream and element index, then Box-Muller in fp64), so the
bits do not depend on numpy's or torch's generator version.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np
from scipy.special import ndtri

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _key(stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        return _mix(np.array([np.uint64(stream & 0xFFFFFFFFFFFFFFFF) * _GOLD + np.uint64(0x1234567)],
                             dtype=np.uint64))[0]


def _uniform_block(key: np.uint64, start: int, count: int, draw: int) -> np.ndarray:
    """Uniforms in [0,1) for counters start..start+count-1 of one stream; draw selects 0/1."""
    with np.errstate(over="ignore"):
        idx = np.arange(start, start + count, dtype=np.uint64)
        h = _mix(key + (idx * np.uint64(2) + np.uint64(draw)) * _GOLD)
    return (h >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def _workers() -> int:
    """Threads used to draw large tensors: the chunks of a counter-based stream are independent, so the
    bits do not depend on this number."""
    try:
        return max(1, min(16, len(os.sched_getaffinity(0))))
    except AttributeError:
        return max(1, min(16, os.cpu_count() or 1))


def _fill(out: np.ndarray, chunk_fn) -> np.ndarray:
    n = out.size
    starts = range(0, n, _CHUNK)

    def one(s):
        c = min(_CHUNK, n - s)
        out[s:s + c] = chunk_fn(s, c)

    if len(starts) <= 1 or _workers() == 1:
        for s in starts:
            one(s)
    else:
        with ThreadPoolExecutor(max_workers=_workers()) as pool:
            list(pool.map(one, starts))
    return out


def uniform(stream: int, n: int) -> np.ndarray:
    """n fp64 uniforms in [0,1)."""
    key = _key(stream)
    return _fill(np.empty(n, dtype=np.float64), lambda s, c: _uniform_block(key, s, c, 0))


def normal(stream: int, n: int) -> np.ndarray:
    """n fp64 standard normals (Box-Muller on two uniforms per element)."""
    key = _key(stream)

    def chunk(s, c):
        u1 = 1.0 - _uniform_block(key, s, c, 0)          # (0,1]
        u2 = _uniform_block(key, s, c, 1)
        return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)

    return _fill(np.empty(n, dtype=np.float64), chunk)


def relu_threshold(p: float) -> float:
    """Shift t with P(z <= t) = p for z ~ N(0,1)."""
    return float(ndtri(p))


def relu_from_normal(z: np.ndarray, p: float) -> np.ndarray:
    """fp32 max(0, z - t) for fp64 standard normals z; p = 0 returns the unclamped Gaussian (no zeros).
    The subtraction and the clamp are done in fp64, then rounded once to fp32."""
    if p <= 0.0:
        return z.astype(np.float32)
    return np.maximum(0.0, z - relu_threshold(p)).astype(np.float32)


def relu_sparse(shape, p: float, stream: int) -> np.ndarray:
    """fp32 tensor max(0, z - t); p = 0 returns the unclamped Gaussian (no zeros).  The normals drawn
    depend on the stream only, not on p: tensors of one stream at several p share their z."""
    return relu_from_normal(normal(stream, int(np.prod(shape))), p).reshape(shape)


def mask_from_uniform(g: np.ndarray, u: np.ndarray, q: float) -> np.ndarray:
    """fp32 g * m for fp64 normals g and uniforms u, m = (u >= q): masked negatives become -0.0."""
    g = g.astype(np.float32)
    if q <= 0.0:
        return g
    return g * (u >= q).astype(np.float32)


def bernoulli_masked(shape, q: float, stream_g: int, stream_m: int) -> np.ndarray:
    """fp32 tensor g * m with m = 1 with probability 1-q.  Masked negatives become -0.0."""
    n = int(np.prod(shape))
    g = normal(stream_g, n)
    if q <= 0.0:
        return g.astype(np.float32).reshape(shape)
    return mask_from_uniform(g, uniform(stream_m, n), q).reshape(shape)


def dead_channels(a: np.ndarray, p_dead: float, stream: int) -> np.ndarray:
    """Copy of an [N][C][H][W] tensor with whole (image, channel) planes set to zero, each with
    probability p_dead: the clustered form ReLU zeros take when a filter does not fire on an image."""
    n, c = a.shape[:2]
    keep = (uniform(stream, n * c) >= p_dead).astype(a.dtype).reshape(n, c, 1, 1)
    return a * keep


def he_normal(shape_kcsr, stream: int) -> np.ndarray:
    """fp32 filters ~ N(0, 2/(C*S*R)) in plain [K][C][S][R] order."""
    k, c, s, r = shape_kcsr
    sigma = np.sqrt(2.0 / (c * s * r))
    return (normal(stream, k * c * s * r) * sigma).astype(np.float32).reshape(shape_kcsr)


def relu_grad(y: np.ndarray, stream_g: int) -> np.ndarray:
    """fp32 tensor g * (y > 0): an upstream Gaussian gradient passed through ReLU'."""
    g = normal(stream_g, y.size).astype(np.float32).reshape(y.shape)
    return g * (np.asarray(y) > 0).astype(np.float32)


def zero_fraction(a: np.ndarray) -> float:
    """Fraction of elements that compare equal to zero (+0 and -0 alike)."""
    return float(np.count_nonzero(a == 0)) / a.size


@dataclass(frozen=True)
class Layer:
    """One convolution workload: shape in the paper's symbols plus target zero fractions."""
    name: str
    N: int
    C: int
    K: int
    H: int
    W: int
    R: int
    S: int
    pad: int
    p_x: float      # target zero fraction of the layer input
    p_dy: float     # target zero fraction of the output gradient
    stride: int = 1

    @property
    def OH(self):
        return (self.H + 2 * self.pad - self.S) // self.stride + 1

    @property
    def OW(self):
        return (self.W + 2 * self.pad - self.R) // self.stride + 1

    @property
    def flops(self):
        return 2 * self.N * self.K * self.C * self.OH * self.OW * self.R * self.S


# Workloads named by the benchmark definition.  vgg*/resnet* shapes are rows of
# the paper's Table 1; zero fractions are the benchmark's.
TINY = Layer("tiny", 1, 16, 16, 8, 8, 3, 3, 1, 0.50, -1.0)          # dy from ReLU' of FWD
VGG3_2_N16 = Layer("vgg3_2", 16, 256, 256, 56, 56, 3, 3, 1, 0.60, 0.50)
RESNET3_2 = Layer("resnet3_2", 32, 128, 128, 28, 28, 3, 3, 1, 0.50, 0.45)
RESNET2_1B = Layer("resnet2_1b", 32, 256, 64, 56, 56, 1, 1, 0, 0.40, 0.50)
RESNET2_2 = Layer("resnet2_2", 32, 64, 64, 56, 56, 3, 3, 1, 0.55, 0.50)
RESNET2_3 = Layer("resnet2_3", 32, 64, 256, 56, 56, 1, 1, 0, 0.55, 0.50)
BOTTLENECK = (RESNET2_1B, RESNET2_2, RESNET2_3)


def vgg16_stack(p: float, n: int = 32):
    """VGG16's non-initial 3x3 layers (Table 1 shapes) at one swept zero fraction."""
    spec = [("vgg1_2", 64, 64, 224), ("vgg2_1", 64, 128, 112), ("vgg2_2", 128, 128, 112),
            ("vgg3_1", 128, 256, 56), ("vgg3_2", 256, 256, 56), ("vgg3_3", 256, 256, 56),
            ("vgg4_1", 256, 512, 28), ("vgg4_2", 512, 512, 28), ("vgg4_3", 512, 512, 28),
            ("vgg5_1", 512, 512, 14), ("vgg5_2", 512, 512, 14), ("vgg5_3", 512, 512, 14)]
    return [Layer(nm, n, c, k, hw, hw, 3, 3, 1, p, p) for nm, c, k, hw in spec]


def table1_layers(n: int = 32, p_x: float = 0.5, p_dy: float = 0.5):
    """Every row of the paper's Table 1 (VGG16 and ResNet-50 v1.5 layer shapes), padding (R-1)/2."""
    spec = [("vgg1_2", 64, 64, 224, 3, 1), ("vgg2_1", 64, 128, 112, 3, 1), ("vgg2_2", 128, 128, 112, 3, 1),
            ("vgg3_1", 128, 256, 56, 3, 1), ("vgg3_2", 256, 256, 56, 3, 1), ("vgg4_1", 256, 512, 28, 3, 1),
            ("vgg4_2", 512, 512, 28, 3, 1), ("vgg5_1", 512, 512, 14, 3, 1), ("resnet2_1a", 64, 64, 56, 1, 1),
            ("resnet2_1b", 256, 64, 56, 1, 1), ("resnet2_2", 64, 64, 56, 3, 1), ("resnet2_3", 64, 256, 56, 1, 1),
            ("resnet3_1a", 256, 128, 56, 1, 1), ("resnet3_1b", 512, 128, 28, 1, 1),
            ("resnet3_2", 128, 128, 28, 3, 1), ("resnet3_2/r", 128, 128, 56, 3, 2),
            ("resnet3_3", 128, 512, 28, 1, 1), ("resnet4_1a", 512, 256, 28, 1, 1),
            ("resnet4_1b", 1024, 256, 14, 1, 1), ("resnet4_2", 256, 256, 14, 3, 1),
            ("resnet4_2/r", 256, 256, 28, 3, 2), ("resnet4_3", 256, 1024, 14, 1, 1),
            ("resnet5_1a", 1024, 512, 14, 1, 1), ("resnet5_1b", 2048, 512, 7, 1, 1),
            ("resnet5_2", 512, 512, 7, 3, 1), ("resnet5_2/r", 512, 512, 14, 3, 2),
            ("resnet5_3", 512, 2048, 7, 1, 1)]
    return [Layer(nm, n, c, k, hw, hw, r, r, (r - 1) // 2, p_x, p_dy, stride)
            for nm, c, k, hw, r, stride in spec]


def make_layer_tensors(layer: Layer, seed: int = 0):
    """(x, w, dy) for a layer in plain layouts, fp32.

    Streams: x = 4*seed, w = 4*seed+1, g = 4*seed+2, m = 4*seed+3.  A layer whose
    p_dy is negative gets no dy here (the caller derives it from a forward
    result with relu_grad and stream 4*seed+2).
    """
    x = relu_sparse((layer.N, layer.C, layer.H, layer.W), layer.p_x, 4 * seed + 0)
    w = he_normal((layer.K, layer.C, layer.S, layer.R), 4 * seed + 1)
    dy = None
    if layer.p_dy >= 0.0:
        dy = bernoulli_masked((layer.N, layer.K, layer.OH, layer.OW), layer.p_dy,
                              4 * seed + 2, 4 * seed + 3)
    return x, w, dy
