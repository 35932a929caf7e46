"""ctypes front end of the group-wise-scale part of the CPU oracle (same C file as the per-row part).

TEST INFRASTRUCTURE ONLY, like fp6_oracle.py.  scales are float16 [M][K/group].
"""
from __future__ import annotations

import ctypes

import numpy as np

from . import fp6_oracle as _six
from .fp6_oracle import _check_shape, _p, _rows_arg, _u16

_ready = False


def _load():
    global _ready
    L = _six._load()
    if not _ready:
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        L.fp6go_quantize.restype = ci
        L.fp6go_quantize.argtypes = [vp, i64, i64, i64, vp, vp]
        L.fp6go_quantize_pack.restype = ci
        L.fp6go_quantize_pack.argtypes = [vp, i64, i64, i64, vp, vp]
        L.fp6go_unpack.restype = ci
        L.fp6go_unpack.argtypes = [vp, vp, i64, i64, i64, vp]
        L.fp6go_linear.restype = ci
        L.fp6go_linear.argtypes = [vp, vp, vp, i64, i64, i64, i64, vp, i64, vp]
        _ready = True
    return L


def quantize(W: np.ndarray, group: int):
    """fp16 W [M][K] -> (codes uint8 [M][K], scales float16 [M][K/group])."""
    Wb = _u16(W)
    M, K = Wb.shape
    assert K % group == 0
    codes = np.empty((M, K), dtype=np.uint8)
    scales = np.empty((M, K // group), dtype=np.uint16)
    if _load().fp6go_quantize(_p(Wb), M, K, group, _p(codes), _p(scales)):
        raise ValueError("W holds inf/NaN")
    return codes, scales.view(np.float16)


def quantize_pack(W: np.ndarray, group: int):
    Wb = _u16(W)
    M, K = Wb.shape
    _check_shape(M, K)
    assert K % group == 0
    packed = np.empty(_six.packed_bytes(M, K), dtype=np.uint8)
    scales = np.empty((M, K // group), dtype=np.uint16)
    rc = _load().fp6go_quantize_pack(_p(Wb), M, K, group, _p(packed), _p(scales))
    if rc == 1:
        raise ValueError("W holds inf/NaN")
    if rc:
        raise MemoryError
    return packed, scales.view(np.float16)


def unpack(packed: np.ndarray, scales: np.ndarray, M: int, K: int, group: int) -> np.ndarray:
    _check_shape(M, K)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    sc = _u16(scales)
    assert packed.size == _six.packed_bytes(M, K) and sc.size == M * (K // group)
    W = np.empty((M, K), dtype=np.uint16)
    if _load().fp6go_unpack(_p(packed), _p(sc), M, K, group, _p(W)):
        raise MemoryError
    return W.view(np.float16)


def linear(packed: np.ndarray, scales: np.ndarray, X: np.ndarray, M: int, K: int, group: int, rows=None) -> np.ndarray:
    _check_shape(M, K)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    Xb = _u16(X)
    N, K2 = Xb.shape
    assert K2 == K
    sc = _u16(scales)
    assert sc.size == M * (K // group)
    r, nrows, rp = _rows_arg(rows, M)
    Y = np.empty((N, nrows), dtype=np.float64)
    if _load().fp6go_linear(_p(packed), _p(sc), _p(Xb), M, N, K, group, rp, nrows, _p(Y)):
        raise MemoryError
    return Y
