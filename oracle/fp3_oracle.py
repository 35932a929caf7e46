"""ctypes front end of the 3-bit (e2m0) part of the CPU oracle (same C file as the 6-bit part).

TEST INFRASTRUCTURE ONLY, like fp6_oracle.py: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg; never by the product package.
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
        L.fp3o_decode.restype = ctypes.c_double
        L.fp3o_decode.argtypes = [ci]
        L.fp3o_scale_for_amax.restype = ctypes.c_uint16
        L.fp3o_scale_for_amax.argtypes = [ctypes.c_uint16]
        L.fp3o_quantize_one.restype = ci
        L.fp3o_quantize_one.argtypes = [ctypes.c_uint16, ctypes.c_uint16]
        L.fp3o_quantize.restype = ci
        L.fp3o_quantize.argtypes = [vp, i64, i64, vp, vp]
        L.fp3o_packed_bytes.restype = i64
        L.fp3o_packed_bytes.argtypes = [i64, i64]
        L.fp3o_pos.restype = ctypes.c_uint64
        L.fp3o_pos.argtypes = [i64, i64, i64, i64, ci]
        L.fp3o_pack.restype = None
        L.fp3o_pack.argtypes = [vp, i64, i64, vp]
        L.fp3o_unpack_codes.restype = None
        L.fp3o_unpack_codes.argtypes = [vp, i64, i64, vp]
        L.fp3o_quantize_pack.restype = ci
        L.fp3o_quantize_pack.argtypes = [vp, i64, i64, vp, vp]
        L.fp3o_unpack.restype = ci
        L.fp3o_unpack.argtypes = [vp, vp, i64, i64, vp]
        L.fp3o_linear_codes.restype = None
        L.fp3o_linear_codes.argtypes = [vp, vp, vp, i64, i64, i64, vp, i64, vp]
        L.fp3o_linear.restype = ci
        L.fp3o_linear.argtypes = [vp, vp, vp, i64, i64, i64, vp, i64, vp]
        _ready = True
    return L


def decode(code: int) -> float:
    return float(_load().fp3o_decode(int(code)))


def decode_table() -> np.ndarray:
    return np.array([decode(c) for c in range(8)], dtype=np.float64)


def scale_for_amax(amax_bits: int) -> int:
    return int(_load().fp3o_scale_for_amax(int(amax_bits)))


def quantize_one(w_bits: int, scale_bits: int) -> int:
    return int(_load().fp3o_quantize_one(int(w_bits), int(scale_bits)))


def pos(M: int, K: int, m: int, k: int, b: int) -> int:
    return int(_load().fp3o_pos(int(M), int(K), int(m), int(k), int(b)))


def packed_bytes(M: int, K: int) -> int:
    return int(_load().fp3o_packed_bytes(int(M), int(K)))


def quantize(W: np.ndarray):
    """fp16 W [M][K] -> (codes uint8 [M][K], scales float16 [M])."""
    Wb = _u16(W)
    M, K = Wb.shape
    codes = np.empty((M, K), dtype=np.uint8)
    scales = np.empty(M, dtype=np.uint16)
    if _load().fp3o_quantize(_p(Wb), M, K, _p(codes), _p(scales)):
        raise ValueError("W holds inf/NaN")
    return codes, scales.view(np.float16)


def pack(codes: np.ndarray) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    M, K = codes.shape
    _check_shape(M, K)
    out = np.empty(packed_bytes(M, K), dtype=np.uint8)
    _load().fp3o_pack(_p(codes), M, K, _p(out))
    return out


def unpack_codes(packed: np.ndarray, M: int, K: int) -> np.ndarray:
    _check_shape(M, K)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.size == packed_bytes(M, K)
    codes = np.empty((M, K), dtype=np.uint8)
    _load().fp3o_unpack_codes(_p(packed), M, K, _p(codes))
    return codes


def quantize_pack(W: np.ndarray):
    """fp16 W [M][K] -> (packed uint8 [3MK/8], scales float16 [M])."""
    Wb = _u16(W)
    M, K = Wb.shape
    _check_shape(M, K)
    packed = np.empty(packed_bytes(M, K), dtype=np.uint8)
    scales = np.empty(M, dtype=np.uint16)
    rc = _load().fp3o_quantize_pack(_p(Wb), M, K, _p(packed), _p(scales))
    if rc == 1:
        raise ValueError("W holds inf/NaN")
    if rc:
        raise MemoryError
    return packed, scales.view(np.float16)


def unpack(packed: np.ndarray, scales: np.ndarray, M: int, K: int) -> np.ndarray:
    _check_shape(M, K)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    sc = _u16(scales)
    assert packed.size == packed_bytes(M, K) and sc.size == M
    W = np.empty((M, K), dtype=np.uint16)
    if _load().fp3o_unpack(_p(packed), _p(sc), M, K, _p(W)):
        raise MemoryError
    return W.view(np.float16)


def linear_codes(codes: np.ndarray, scales: np.ndarray, X: np.ndarray, rows=None) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    M, K = codes.shape
    Xb = _u16(X)
    N, K2 = Xb.shape
    assert K2 == K
    sc = _u16(scales)
    r, nrows, rp = _rows_arg(rows, M)
    Y = np.empty((N, nrows), dtype=np.float64)
    _load().fp3o_linear_codes(_p(codes), _p(sc), _p(Xb), M, N, K, rp, nrows, _p(Y))
    return Y


def linear(packed: np.ndarray, scales: np.ndarray, X: np.ndarray, M: int, K: int, rows=None) -> np.ndarray:
    _check_shape(M, K)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.size == packed_bytes(M, K)
    Xb = _u16(X)
    N, K2 = Xb.shape
    assert K2 == K
    sc = _u16(scales)
    assert sc.size == M
    r, nrows, rp = _rows_arg(rows, M)
    Y = np.empty((N, nrows), dtype=np.float64)
    if _load().fp3o_linear(_p(packed), _p(sc), _p(Xb), M, N, K, rp, nrows, _p(Y)):
        raise MemoryError
    return Y
