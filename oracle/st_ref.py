"""ctypes front end of the CPU oracle (oracle/st_ref_conv.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  Nothing in the GPU package imports this module,
and this module imports nothing from the GPU package.

All tensors are plain row-major numpy arrays (x[N][C][H][W], w[K][C][S][R],
y[N][K][OH][OW]); see the header of st_ref_conv.c for the definitions
(SparseTrain Sec. 2.1, Eq. (1) and the passage after Eq. (2); Alg. 1 and 4).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "st_ref_conv.c")
_LIB = os.path.join(_HERE, "libst_ref.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math) and return the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-fno-fast-math", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        i64p = ctypes.POINTER(ctypes.c_int64)
        for name in ("st_ref_conv_fwd", "st_ref_conv_bwi", "st_ref_conv_bww"):
            fn = getattr(lib, name)
            fn.argtypes = [i32p, f32p, f32p, f64p, f64p]
            fn.restype = ctypes.c_int
        for name in ("st_ref_conv_fwd_at", "st_ref_conv_bwi_at", "st_ref_conv_bww_at"):
            fn = getattr(lib, name)
            fn.argtypes = [i32p, f32p, f32p, ctypes.c_int64, i32p, f64p, f64p]
            fn.restype = ctypes.c_int
        for name in ("st_ref_conv_fwd_scatter", "st_ref_conv_bwi_scatter"):
            fn = getattr(lib, name)
            fn.argtypes = [i32p, f32p, f32p, f64p, i64p]
            fn.restype = ctypes.c_int
        lib.st_ref_conv_bww_scatter.argtypes = [i32p, f32p, f32p, ctypes.c_int, f64p, i64p]
        lib.st_ref_conv_bww_scatter.restype = ctypes.c_int
        lib.st_ref_out_dims.argtypes = [i32p, i32p, i32p]
        lib.st_ref_out_dims.restype = ctypes.c_int
        lib.st_ref_threads.argtypes = []
        lib.st_ref_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


@dataclass(frozen=True)
class Geom:
    """Convolution geometry in the paper's symbols (Table 1).

    R is the filter width (pairs with W), S the filter height (pairs with H);
    stride_w = O, stride_h = P.  Padding is symmetric per axis.
    """
    N: int
    C: int
    K: int
    H: int
    W: int
    R: int
    S: int
    stride_w: int = 1
    stride_h: int = 1
    pad_w: int = 0
    pad_h: int = 0

    @property
    def OH(self) -> int:
        return (self.H + 2 * self.pad_h - self.S) // self.stride_h + 1

    @property
    def OW(self) -> int:
        return (self.W + 2 * self.pad_w - self.R) // self.stride_w + 1

    @property
    def x_shape(self):
        return (self.N, self.C, self.H, self.W)

    @property
    def y_shape(self):
        return (self.N, self.K, self.OH, self.OW)

    @property
    def w_shape(self):
        return (self.K, self.C, self.S, self.R)

    @property
    def flops(self) -> int:
        """Dense-equivalent flop count of one pass, padded taps included."""
        return 2 * self.N * self.K * self.C * self.OH * self.OW * self.R * self.S

    def dims(self) -> np.ndarray:
        return np.array([self.N, self.C, self.K, self.H, self.W, self.R, self.S,
                         self.stride_w, self.stride_h, self.pad_w, self.pad_h], dtype=np.int32)


def threads() -> int:
    return int(_load().st_ref_threads())


def _f32(a, shape):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _check(rc, name):
    if rc != 0:
        raise ValueError(f"{name} failed with code {rc}")


def _gather(name, g: Geom, a, a_shape, b, b_shape, out_shape):
    lib = _load()
    a = _f32(a, a_shape)
    b = _f32(b, b_shape)
    out = np.empty(out_shape, dtype=np.float64)
    out_abs = np.empty(out_shape, dtype=np.float64)
    d = g.dims()
    rc = getattr(lib, name)(_ptr(d, ctypes.c_int32), _ptr(a, ctypes.c_float), _ptr(b, ctypes.c_float),
                            _ptr(out, ctypes.c_double), _ptr(out_abs, ctypes.c_double))
    _check(rc, name)
    return out, out_abs


def conv_fwd(g: Geom, x, w):
    """Eq. (1).  Returns (y, sum|terms|), both fp64, shape [N][K][OH][OW]."""
    return _gather("st_ref_conv_fwd", g, x, g.x_shape, w, g.w_shape, g.y_shape)


def conv_bwi(g: Geom, dy, w):
    """Gradient w.r.t. the input (Sec. 2.1).  Returns (dx, sum|terms|), [N][C][H][W]."""
    return _gather("st_ref_conv_bwi", g, dy, g.y_shape, w, g.w_shape, g.x_shape)


def conv_bww(g: Geom, x, dy):
    """Gradient w.r.t. the filters (Sec. 2.1).  Returns (dw, sum|terms|), [K][C][S][R]."""
    return _gather("st_ref_conv_bww", g, x, g.x_shape, dy, g.y_shape, g.w_shape)


def _sampled(name, g: Geom, a, a_shape, b, b_shape, coords):
    lib = _load()
    a = _f32(a, a_shape)
    b = _f32(b, b_shape)
    coords = np.ascontiguousarray(coords, dtype=np.int32)
    if coords.ndim != 2 or coords.shape[1] != 4:
        raise ValueError("coords must have shape [n_samples][4]")
    n = coords.shape[0]
    out = np.empty(n, dtype=np.float64)
    out_abs = np.empty(n, dtype=np.float64)
    d = g.dims()
    rc = getattr(lib, name)(_ptr(d, ctypes.c_int32), _ptr(a, ctypes.c_float), _ptr(b, ctypes.c_float),
                            ctypes.c_int64(n), _ptr(coords, ctypes.c_int32),
                            _ptr(out, ctypes.c_double), _ptr(out_abs, ctypes.c_double))
    _check(rc, name)
    return out, out_abs


def conv_fwd_at(g: Geom, x, w, coords):
    """Eq. (1) at the sampled output coordinates (n,k,oh,ow)."""
    return _sampled("st_ref_conv_fwd_at", g, x, g.x_shape, w, g.w_shape, coords)


def conv_bwi_at(g: Geom, dy, w, coords):
    """BWI at the sampled coordinates (n,c,ih,iw)."""
    return _sampled("st_ref_conv_bwi_at", g, dy, g.y_shape, w, g.w_shape, coords)


def conv_bww_at(g: Geom, x, dy, coords):
    """BWW at the sampled coordinates (k,c,v,u)."""
    return _sampled("st_ref_conv_bww_at", g, x, g.x_shape, dy, g.y_shape, coords)


def conv_fwd_scatter(g: Geom, x, w):
    """Alg. 1 with the zero test.  Returns (y fp64, number of skipped input elements)."""
    lib = _load()
    x = _f32(x, g.x_shape)
    w = _f32(w, g.w_shape)
    y = np.empty(g.y_shape, dtype=np.float64)
    skipped = ctypes.c_int64(0)
    d = g.dims()
    rc = lib.st_ref_conv_fwd_scatter(_ptr(d, ctypes.c_int32), _ptr(x, ctypes.c_float),
                                     _ptr(w, ctypes.c_float), _ptr(y, ctypes.c_double),
                                     ctypes.byref(skipped))
    _check(rc, "st_ref_conv_fwd_scatter")
    return y, int(skipped.value)


def conv_bwi_scatter(g: Geom, dy, w):
    """Input-stationary BWI with the zero test on dy.  Returns (dx fp64, skipped count)."""
    lib = _load()
    dy = _f32(dy, g.y_shape)
    w = _f32(w, g.w_shape)
    dx = np.empty(g.x_shape, dtype=np.float64)
    skipped = ctypes.c_int64(0)
    d = g.dims()
    rc = lib.st_ref_conv_bwi_scatter(_ptr(d, ctypes.c_int32), _ptr(dy, ctypes.c_float),
                                     _ptr(w, ctypes.c_float), _ptr(dx, ctypes.c_double),
                                     ctypes.byref(skipped))
    _check(rc, "st_ref_conv_bwi_scatter")
    return dx, int(skipped.value)


def conv_bww_scatter(g: Geom, x, dy, test_dy: bool = False):
    """Alg. 4 with the zero test on x (or on dy).  Returns (dw fp64, skipped count)."""
    lib = _load()
    x = _f32(x, g.x_shape)
    dy = _f32(dy, g.y_shape)
    dw = np.empty(g.w_shape, dtype=np.float64)
    skipped = ctypes.c_int64(0)
    d = g.dims()
    rc = lib.st_ref_conv_bww_scatter(_ptr(d, ctypes.c_int32), _ptr(x, ctypes.c_float),
                                     _ptr(dy, ctypes.c_float), ctypes.c_int(1 if test_dy else 0),
                                     _ptr(dw, ctypes.c_double), ctypes.byref(skipped))
    _check(rc, "st_ref_conv_bww_scatter")
    return dw, int(skipped.value)


def rel_err(got, ref, ref_abs):
    """Per-element |got - ref| / sum|terms|; where sum|terms| is 0 the result must be exactly 0.

    Returns (max relative error over elements with a non-zero scale,
             number of elements whose scale is 0 but whose value is not).
    A non-finite element of got counts as an infinite error (scale > 0) or as a bad zero (scale 0).
    Pinned by tests/test_oracle_pins.py::test_rel_err_* (hand-computed cases, planted deviations).
    """
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    ref_abs = np.asarray(ref_abs, dtype=np.float64)
    if got.shape != ref.shape or ref.shape != ref_abs.shape:
        raise ValueError(f"shape mismatch: got {got.shape}, ref {ref.shape}, scale {ref_abs.shape}")
    nz = ref_abs > 0
    err = 0.0
    if nz.any():
        e = np.abs(got[nz] - ref[nz]) / ref_abs[nz]
        err = float("inf") if not np.isfinite(e).all() else float(np.max(e))
    bad_zero = int(np.count_nonzero(~(got[~nz] == 0.0)))
    return err, bad_zero
