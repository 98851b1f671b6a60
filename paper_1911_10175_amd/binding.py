"""ctypes binding of libst_conv.so.  Argument marshalling only.

The functions carry the names of the C entry points (include/st_conv.h) and take anything
with a ``data_ptr()`` method (torch tensors on the GPU) or a raw integer device address.
There is no CPU fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

ST_PASS_FWD, ST_PASS_BWI, ST_PASS_BWW, ST_PASS_BWW_DY, ST_PASS_BWW_AUTO = 0, 1, 2, 3, 4
ST_PASS_FWD_AUTO, ST_PASS_BWI_AUTO = 5, 6
ST_OK = 0

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libst_conv.so"
EXPORTS = ("st_conv_fwd", "st_conv_fwd_dense", "st_conv_bwi", "st_conv_bwi_dense", "st_conv_bww",
           "st_conv_bww_dense", "st_conv_bww_dy", "st_conv_bww_auto", "st_conv_fwd_auto", "st_conv_bwi_auto",
           "st_conv_workspace_bytes", "st_conv_sparse_threshold", "st_status_str", "st_conv_version",
           "st_conv_fwd_static", "st_conv_kernel_name", "st_probe_issue_rate")


class StConvError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"st_conv status {status}: {message}")
        self.status = status


class _CDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "C", "K", "H", "W", "R", "S", "stride_w", "stride_h", "pad_w", "pad_h")]


@dataclass(frozen=True)
class ConvDesc:
    """st_conv_desc: R is the filter width (pairs with W), S the filter height (pairs with H)."""
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
    def flops(self) -> int:
        return 2 * self.N * self.K * self.C * self.OH * self.OW * self.R * self.S

    def _c(self) -> _CDesc:
        return _CDesc(self.N, self.C, self.K, self.H, self.W, self.R, self.S,
                      self.stride_w, self.stride_h, self.pad_w, self.pad_h)


def lib_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


_lib = None


def load_library():
    """Load libst_conv.so from the package directory; raises if it has not been built."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise FileNotFoundError(
                f"{path} not found: build it first (python -c 'import __graft_entry__ as g; g.build()' "
                f"or make -C paper_1911_10175_amd/csrc).  There is no fallback path.")
        lib = ctypes.CDLL(path)
        p = ctypes.c_void_p
        for name in EXPORTS[:10]:
            fn = getattr(lib, name)
            fn.argtypes = [ctypes.POINTER(_CDesc), p, p, p, p, ctypes.c_size_t, p]
            fn.restype = ctypes.c_int
        lib.st_conv_fwd_static.argtypes = [ctypes.POINTER(_CDesc), p, p, p, p]
        lib.st_conv_fwd_static.restype = ctypes.c_int
        lib.st_conv_kernel_name.argtypes = [ctypes.POINTER(_CDesc), ctypes.c_int, ctypes.c_char_p, ctypes.c_size_t]
        lib.st_conv_kernel_name.restype = ctypes.c_int
        lib.st_probe_issue_rate.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, p, p]
        lib.st_probe_issue_rate.restype = ctypes.c_int
        lib.st_conv_workspace_bytes.argtypes = [ctypes.POINTER(_CDesc), ctypes.c_int, ctypes.c_int]
        lib.st_conv_workspace_bytes.restype = ctypes.c_size_t
        lib.st_conv_sparse_threshold.argtypes = [ctypes.POINTER(_CDesc), ctypes.c_int]
        lib.st_conv_sparse_threshold.restype = ctypes.c_int
        lib.st_status_str.argtypes = [ctypes.c_int]
        lib.st_status_str.restype = ctypes.c_char_p
        lib.st_conv_version.argtypes = []
        lib.st_conv_version.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def _addr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _nbytes(t) -> int:
    if t is None or isinstance(t, int):
        return 0
    return t.numel() * t.element_size()


def _stream(stream):
    if stream is None:
        return None
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)     # torch.cuda.Stream


def st_status_str(status: int) -> str:
    return load_library().st_status_str(int(status)).decode()


def st_conv_version() -> str:
    return load_library().st_conv_version().decode()


def st_conv_sparse_threshold(desc: ConvDesc, conv_pass: int) -> int:
    c = desc._c()
    return int(load_library().st_conv_sparse_threshold(ctypes.byref(c), int(conv_pass)))


def st_conv_workspace_bytes(desc: ConvDesc, conv_pass: int, dense: bool = False) -> int:
    c = desc._c()
    return int(load_library().st_conv_workspace_bytes(ctypes.byref(c), int(conv_pass), 1 if dense else 0))


def _call(name, desc, a, b, out, ws, ws_bytes, stream, check):
    lib = load_library()
    c = desc._c()
    if ws_bytes is None:
        ws_bytes = _nbytes(ws)
    rc = getattr(lib, name)(ctypes.byref(c), _addr(a), _addr(b), _addr(out), _addr(ws),
                            ctypes.c_size_t(ws_bytes), _stream(stream))
    if check and rc != ST_OK:
        raise StConvError(rc, st_status_str(rc))
    return rc


def st_conv_fwd(desc, x, w, y, ws=None, stream=None, ws_bytes=None, check=True):
    return _call("st_conv_fwd", desc, x, w, y, ws, ws_bytes, stream, check)


def st_conv_fwd_dense(desc, x, w, y, ws=None, stream=None, ws_bytes=None, check=True):
    return _call("st_conv_fwd_dense", desc, x, w, y, ws, ws_bytes, stream, check)


def st_conv_bwi(desc, dy, w, dx, ws=None, stream=None, ws_bytes=None, check=True):
    return _call("st_conv_bwi", desc, dy, w, dx, ws, ws_bytes, stream, check)


def st_conv_bwi_dense(desc, dy, w, dx, ws=None, stream=None, ws_bytes=None, check=True):
    return _call("st_conv_bwi_dense", desc, dy, w, dx, ws, ws_bytes, stream, check)


def st_conv_bww(desc, x, dy, dw, ws=None, stream=None, ws_bytes=None, check=True):
    return _call("st_conv_bww", desc, x, dy, dw, ws, ws_bytes, stream, check)


def st_conv_bww_dense(desc, x, dy, dw, ws=None, stream=None, ws_bytes=None, check=True):
    return _call("st_conv_bww_dense", desc, x, dy, dw, ws, ws_bytes, stream, check)


def st_conv_bww_dy(desc, x, dy, dw, ws=None, stream=None, ws_bytes=None, check=True):
    return _call("st_conv_bww_dy", desc, x, dy, dw, ws, ws_bytes, stream, check)


def st_conv_bww_auto(desc, x, dy, dw, ws=None, stream=None, ws_bytes=None, check=True):
    return _call("st_conv_bww_auto", desc, x, dy, dw, ws, ws_bytes, stream, check)


def st_conv_fwd_auto(desc, x, w, y, ws=None, stream=None, ws_bytes=None, check=True):
    return _call("st_conv_fwd_auto", desc, x, w, y, ws, ws_bytes, stream, check)


def st_conv_bwi_auto(desc, dy, w, dx, ws=None, stream=None, ws_bytes=None, check=True):
    return _call("st_conv_bwi_auto", desc, dy, w, dx, ws, ws_bytes, stream, check)


def st_conv_fwd_static(desc, x, w, y, stream=None, check=True):
    """st_conv_fwd without a workspace argument (built-in 16 MiB scratch; allocates nothing)."""
    lib = load_library()
    c = desc._c()
    rc = lib.st_conv_fwd_static(ctypes.byref(c), _addr(x), _addr(w), _addr(y), _stream(stream))
    if check and rc != ST_OK:
        raise StConvError(rc, st_status_str(rc))
    return rc


def st_conv_kernel_name(desc, conv_pass: int):
    """Name of the kernel instance st_conv_fwd / st_conv_bwi launches for this geometry, or None where the
    library has no name to give (other passes, geometries served by the generic kernels)."""
    c = desc._c()
    buf = ctypes.create_string_buffer(128)
    rc = load_library().st_conv_kernel_name(ctypes.byref(c), int(conv_pass), buf, 128)
    return buf.value.decode() if rc == ST_OK else None


def st_probe_issue_rate(pattern: int, workgroups: int, iters: int, out, stream=None, check=True):
    """Measurement aid: bare v_fmac_f32 / MFMA instruction streams (see include/st_conv.h)."""
    rc = load_library().st_probe_issue_rate(int(pattern), int(workgroups), int(iters), _addr(out), _stream(stream))
    if check and rc != ST_OK:
        raise StConvError(rc, st_status_str(rc))
    return rc
