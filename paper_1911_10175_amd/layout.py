"""Index permutations between plain tensors and the library's blocked layouts.

No arithmetic: only reshape / permute.  Works on numpy arrays and torch tensors alike.

  activations  plain [N][C][H][W]      <->  blocked [N][C/16][H][W][16]
  filters      plain [K][C][S][R]      <->  blocked [K/16][C/16][S][R][16 c][16 k]
"""
from __future__ import annotations

import numpy as np

B = 16


def _is_np(a):
    return isinstance(a, np.ndarray)


def _permute(a, order):
    return a.transpose(order) if _is_np(a) else a.permute(*order)


def _contig(a):
    return np.ascontiguousarray(a) if _is_np(a) else a.contiguous()


def pack_activations(a):
    n, c, h, w = a.shape
    if c % B:
        raise ValueError("channel count must be a multiple of 16")
    return _contig(_permute(a.reshape(n, c // B, B, h, w), (0, 1, 3, 4, 2)))


def unpack_activations(a):
    n, cb, h, w, b = a.shape
    if b != B:
        raise ValueError("last dimension must be 16")
    return _contig(_permute(a, (0, 1, 4, 2, 3))).reshape(n, cb * B, h, w)


def pack_filters(f):
    k, c, s, r = f.shape
    if k % B or c % B:
        raise ValueError("K and C must be multiples of 16")
    # [kb][ki][cb][ci][s][r] -> [kb][cb][s][r][ci][ki]
    return _contig(_permute(f.reshape(k // B, B, c // B, B, s, r), (0, 2, 4, 5, 3, 1)))


def unpack_filters(f):
    kb, cb, s, r, ci, ki = f.shape
    if ci != B or ki != B:
        raise ValueError("last two dimensions must be 16")
    # [kb][cb][s][r][ci][ki] -> [kb][ki][cb][ci][s][r]
    return _contig(_permute(f, (0, 5, 1, 4, 2, 3))).reshape(kb * B, cb * B, s, r)
