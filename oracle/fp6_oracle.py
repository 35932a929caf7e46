"""ctypes front end of the CPU oracle (fp6_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports it, and this
module never imports the product package.

All arrays are numpy, host memory.  fp16 data travels as uint16 bit patterns or
as float16 arrays (viewed as uint16 here).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "fp6_oracle.c"
_LIB = _HERE / "libfp6_oracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile fp6_oracle.c with gcc (OpenMP over output rows)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
             "-o", str(tmp), str(_SRC), "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = ctypes.CDLL(str(_LIB))
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    L.fp6o_half_to_double.restype = ctypes.c_double
    L.fp6o_half_to_double.argtypes = [ctypes.c_uint16]
    L.fp6o_double_to_half.restype = ctypes.c_uint16
    L.fp6o_double_to_half.argtypes = [ctypes.c_double]
    L.fp6o_decode.restype = ctypes.c_double
    L.fp6o_decode.argtypes = [ci]
    L.fp6o_scale_for_amax.restype = ctypes.c_uint16
    L.fp6o_scale_for_amax.argtypes = [ctypes.c_uint16]
    L.fp6o_quantize_one.restype = ci
    L.fp6o_quantize_one.argtypes = [ctypes.c_uint16, ctypes.c_uint16]
    L.fp6o_quantize.restype = ci
    L.fp6o_quantize.argtypes = [vp, i64, i64, vp, vp]
    L.fp6o_packed_bytes.restype = i64
    L.fp6o_packed_bytes.argtypes = [i64, i64]
    L.fp6o_pos.restype = ctypes.c_uint64
    L.fp6o_pos.argtypes = [i64, i64, i64, i64, ci]
    L.fp6o_pack.restype = None
    L.fp6o_pack.argtypes = [vp, i64, i64, vp]
    L.fp6o_unpack_codes.restype = None
    L.fp6o_unpack_codes.argtypes = [vp, i64, i64, vp]
    L.fp6o_quantize_pack.restype = ci
    L.fp6o_quantize_pack.argtypes = [vp, i64, i64, vp, vp]
    L.fp6o_unpack.restype = ci
    L.fp6o_unpack.argtypes = [vp, vp, i64, i64, vp]
    L.fp6o_linear_codes.restype = None
    L.fp6o_linear_codes.argtypes = [vp, vp, vp, i64, i64, i64, vp, i64, vp]
    L.fp6o_linear.restype = ci
    L.fp6o_linear.argtypes = [vp, vp, vp, i64, i64, i64, vp, i64, vp]
    L.fp6o_linear_fused.restype = ci
    L.fp6o_linear_fused.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp, ci, vp, i64, vp]
    L.fpxo_linear_fused.restype = ci
    L.fpxo_linear_fused.argtypes = [ci, i64, vp, vp, vp, i64, i64, i64, vp, vp, ci, vp, i64, vp]
    L.fp6o_linear_f16.restype = None
    L.fp6o_linear_f16.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp]
    L.fp6o_threads.restype = ci
    L.fp6o_threads.argtypes = []
    _lib = L
    return L


def _u16(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("fp16 data must be float16 or uint16 bit patterns, got %s" % a.dtype)
    return a


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _check_shape(M: int, K: int):
    if M <= 0 or K <= 0 or M % 16 or K % 256:
        raise ValueError("oracle layout needs M %% 16 == 0 and K %% 256 == 0, got M=%d K=%d" % (M, K))


# --------------------------------------------------------------- scalars ----
def threads() -> int:
    return int(_load().fp6o_threads())


def half_to_double(bits: int) -> float:
    return float(_load().fp6o_half_to_double(int(bits)))


def double_to_half(x: float) -> int:
    return int(_load().fp6o_double_to_half(float(x)))


def decode(code: int) -> float:
    return float(_load().fp6o_decode(int(code)))


def decode_table() -> np.ndarray:
    return np.array([decode(c) for c in range(64)], dtype=np.float64)


def scale_for_amax(amax_bits: int) -> int:
    return int(_load().fp6o_scale_for_amax(int(amax_bits)))


def quantize_one(w_bits: int, scale_bits: int) -> int:
    return int(_load().fp6o_quantize_one(int(w_bits), int(scale_bits)))


def pos(M: int, K: int, m: int, k: int, b: int) -> int:
    return int(_load().fp6o_pos(int(M), int(K), int(m), int(k), int(b)))


def packed_bytes(M: int, K: int) -> int:
    return int(_load().fp6o_packed_bytes(int(M), int(K)))


# ---------------------------------------------------------------- arrays ----
def quantize(W: np.ndarray):
    """fp16 W [M][K] -> (codes uint8 [M][K], scales float16 [M])."""
    Wb = _u16(W)
    M, K = Wb.shape
    codes = np.empty((M, K), dtype=np.uint8)
    scales = np.empty(M, dtype=np.uint16)
    rc = _load().fp6o_quantize(_p(Wb), M, K, _p(codes), _p(scales))
    if rc:
        raise ValueError("W holds inf/NaN")
    return codes, scales.view(np.float16)


def pack(codes: np.ndarray) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    M, K = codes.shape
    _check_shape(M, K)
    out = np.empty(packed_bytes(M, K), dtype=np.uint8)
    _load().fp6o_pack(_p(codes), M, K, _p(out))
    return out


def unpack_codes(packed: np.ndarray, M: int, K: int) -> np.ndarray:
    _check_shape(M, K)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.size == packed_bytes(M, K)
    codes = np.empty((M, K), dtype=np.uint8)
    _load().fp6o_unpack_codes(_p(packed), M, K, _p(codes))
    return codes


def quantize_pack(W: np.ndarray):
    """fp16 W [M][K] -> (packed uint8 [3MK/4], scales float16 [M])."""
    Wb = _u16(W)
    M, K = Wb.shape
    _check_shape(M, K)
    packed = np.empty(packed_bytes(M, K), dtype=np.uint8)
    scales = np.empty(M, dtype=np.uint16)
    rc = _load().fp6o_quantize_pack(_p(Wb), M, K, _p(packed), _p(scales))
    if rc == 1:
        raise ValueError("W holds inf/NaN")
    if rc:
        raise MemoryError
    return packed, scales.view(np.float16)


def unpack(packed: np.ndarray, scales: np.ndarray, M: int, K: int) -> np.ndarray:
    """packed + scales -> float16 [M][K]."""
    _check_shape(M, K)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    sc = _u16(scales)
    assert packed.size == packed_bytes(M, K) and sc.size == M
    W = np.empty((M, K), dtype=np.uint16)
    if _load().fp6o_unpack(_p(packed), _p(sc), M, K, _p(W)):
        raise MemoryError
    return W.view(np.float16)


def _rows_arg(rows, M):
    if rows is None:
        return None, M, ctypes.c_void_p(0)
    r = np.ascontiguousarray(rows, dtype=np.int64)
    assert r.ndim == 1 and r.size > 0 and r.min() >= 0 and r.max() < M
    return r, r.size, _p(r)


def linear_codes(codes: np.ndarray, scales: np.ndarray, X: np.ndarray, rows=None) -> np.ndarray:
    """Y[n][i] (float64) for codes [M][K], scales [M], X fp16 [N][K]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    M, K = codes.shape
    Xb = _u16(X)
    N, K2 = Xb.shape
    assert K2 == K
    sc = _u16(scales)
    r, nrows, rp = _rows_arg(rows, M)
    Y = np.empty((N, nrows), dtype=np.float64)
    _load().fp6o_linear_codes(_p(codes), _p(sc), _p(Xb), M, N, K, rp, nrows, _p(Y))
    return Y


def linear(packed: np.ndarray, scales: np.ndarray, X: np.ndarray, M: int, K: int, rows=None) -> np.ndarray:
    """Y[n][i] (float64) from the packed stream; rows=None means all M rows."""
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
    if _load().fp6o_linear(_p(packed), _p(sc), _p(Xb), M, N, K, rp, nrows, _p(Y)):
        raise MemoryError
    return Y


def linear_fused(packed: np.ndarray, scales: np.ndarray, X: np.ndarray, M: int, K: int, bias=None,
                 residual=None, gated: bool = False, rows=None, bits: int = 6, group: int = 0) -> np.ndarray:
    """The linear layer plus bias / silu(gate)*up / residual (see fp6o_linear_fused); float64 [N][nrows].

    rows lists OUTPUT rows (of M/2 when gated); bias fp16 [M]; residual fp16 [N][Mout].  bits = 5, 4, 3
    takes the packed stream of that width; bits = 6 with group > 0 takes scales [M][K/group]."""
    _check_shape(M, K)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.size == M * K * bits // 8
    Xb = _u16(X)
    N, K2 = Xb.shape
    assert K2 == K
    sc = _u16(scales)
    assert sc.size == (M * (K // group) if group else M)
    Mout = M // 2 if gated else M
    null = ctypes.c_void_p(0)
    bp = rp_ = null
    if bias is not None:
        bb = _u16(bias)
        assert bb.shape == (M,)
        bp = _p(bb)
    if residual is not None:
        rb = _u16(residual)
        assert rb.shape == (N, Mout)
        rp_ = _p(rb)
    r, nrows, rp = _rows_arg(rows, Mout)
    Y = np.empty((N, nrows), dtype=np.float64)
    rc = _load().fpxo_linear_fused(int(bits), int(group), _p(packed), _p(sc), _p(Xb), M, N, K, bp, rp_,
                                   int(bool(gated)), rp, nrows, _p(Y))
    if rc == 2:
        raise MemoryError
    if rc:
        raise ValueError("gated needs an even M; bits must be 3..6; group only with 6 bits")
    return Y


def linear_f16(W: np.ndarray, X: np.ndarray, rows=None) -> np.ndarray:
    """Y[n][i] = sum_k W[m][k] X[n][k] in float64, fp16 inputs (W16A16 comparison)."""
    Wb = _u16(W)
    M, K = Wb.shape
    Xb = _u16(X)
    N, K2 = Xb.shape
    assert K2 == K
    r, nrows, rp = _rows_arg(rows, M)
    Y = np.empty((N, nrows), dtype=np.float64)
    _load().fp6o_linear_f16(_p(Wb), _p(Xb), M, N, K, rp, nrows, _p(Y))
    return Y
