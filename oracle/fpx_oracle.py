"""ctypes front end of the 5-, 4- and 3-bit parts of the CPU oracle (same C file as the 6-bit part): one
class over the C functions `<prefix>o_*`, one instance per width.

TEST INFRASTRUCTURE ONLY, like fp6_oracle.py: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg; never by the product package.
"""
from __future__ import annotations

import ctypes

import numpy as np

from . import fp6_oracle as _six
from .fp6_oracle import _check_shape, _p, _rows_arg, _u16


class NarrowOracle:
    """The oracle of one weight width: `prefix` names the C functions, `bits` the code width."""

    def __init__(self, prefix: str, bits: int, fmt: str):
        self.prefix, self.bits, self.fmt = prefix, bits, fmt
        self.n_codes = 1 << bits
        self._ready = False

    def _f(self, name: str):
        L = _six._load()
        if not self._ready:
            i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
            sig = {
                "decode": (ctypes.c_double, [ci]),
                "scale_for_amax": (ctypes.c_uint16, [ctypes.c_uint16]),
                "quantize_one": (ci, [ctypes.c_uint16, ctypes.c_uint16]),
                "quantize": (ci, [vp, i64, i64, vp, vp]),
                "packed_bytes": (i64, [i64, i64]),
                "pos": (ctypes.c_uint64, [i64, i64, i64, i64, ci]),
                "pack": (None, [vp, i64, i64, vp]),
                "unpack_codes": (None, [vp, i64, i64, vp]),
                "quantize_pack": (ci, [vp, i64, i64, vp, vp]),
                "unpack": (ci, [vp, vp, i64, i64, vp]),
                "linear_codes": (None, [vp, vp, vp, i64, i64, i64, vp, i64, vp]),
                "linear": (ci, [vp, vp, vp, i64, i64, i64, vp, i64, vp]),
            }
            for fn, (res, args) in sig.items():
                f = getattr(L, "%so_%s" % (self.prefix, fn))
                f.restype, f.argtypes = res, args
            self._ready = True
        return getattr(L, "%so_%s" % (self.prefix, name))

    def decode(self, code: int) -> float:
        return float(self._f("decode")(int(code)))

    def decode_table(self) -> np.ndarray:
        return np.array([self.decode(c) for c in range(self.n_codes)], dtype=np.float64)

    def scale_for_amax(self, amax_bits: int) -> int:
        return int(self._f("scale_for_amax")(int(amax_bits)))

    def quantize_one(self, w_bits: int, scale_bits: int) -> int:
        return int(self._f("quantize_one")(int(w_bits), int(scale_bits)))

    def pos(self, M: int, K: int, m: int, k: int, b: int) -> int:
        return int(self._f("pos")(int(M), int(K), int(m), int(k), int(b)))

    def packed_bytes(self, M: int, K: int) -> int:
        return int(self._f("packed_bytes")(int(M), int(K)))

    def quantize(self, W: np.ndarray):
        """fp16 W [M][K] -> (codes uint8 [M][K], scales float16 [M])."""
        Wb = _u16(W)
        M, K = Wb.shape
        codes = np.empty((M, K), dtype=np.uint8)
        scales = np.empty(M, dtype=np.uint16)
        if self._f("quantize")(_p(Wb), M, K, _p(codes), _p(scales)):
            raise ValueError("W holds inf/NaN")
        return codes, scales.view(np.float16)

    def pack(self, codes: np.ndarray) -> np.ndarray:
        codes = np.ascontiguousarray(codes, dtype=np.uint8)
        M, K = codes.shape
        _check_shape(M, K)
        out = np.empty(self.packed_bytes(M, K), dtype=np.uint8)
        self._f("pack")(_p(codes), M, K, _p(out))
        return out

    def unpack_codes(self, packed: np.ndarray, M: int, K: int) -> np.ndarray:
        _check_shape(M, K)
        packed = np.ascontiguousarray(packed, dtype=np.uint8)
        assert packed.size == self.packed_bytes(M, K)
        codes = np.empty((M, K), dtype=np.uint8)
        self._f("unpack_codes")(_p(packed), M, K, _p(codes))
        return codes

    def quantize_pack(self, W: np.ndarray):
        """fp16 W [M][K] -> (packed uint8 [bits*M*K/8], scales float16 [M])."""
        Wb = _u16(W)
        M, K = Wb.shape
        _check_shape(M, K)
        packed = np.empty(self.packed_bytes(M, K), dtype=np.uint8)
        scales = np.empty(M, dtype=np.uint16)
        rc = self._f("quantize_pack")(_p(Wb), M, K, _p(packed), _p(scales))
        if rc == 1:
            raise ValueError("W holds inf/NaN")
        if rc:
            raise MemoryError
        return packed, scales.view(np.float16)

    def unpack(self, packed: np.ndarray, scales: np.ndarray, M: int, K: int) -> np.ndarray:
        _check_shape(M, K)
        packed = np.ascontiguousarray(packed, dtype=np.uint8)
        sc = _u16(scales)
        assert packed.size == self.packed_bytes(M, K) and sc.size == M
        W = np.empty((M, K), dtype=np.uint16)
        if self._f("unpack")(_p(packed), _p(sc), M, K, _p(W)):
            raise MemoryError
        return W.view(np.float16)

    def linear_codes(self, codes: np.ndarray, scales: np.ndarray, X: np.ndarray, rows=None) -> np.ndarray:
        codes = np.ascontiguousarray(codes, dtype=np.uint8)
        M, K = codes.shape
        Xb = _u16(X)
        N, K2 = Xb.shape
        assert K2 == K
        sc = _u16(scales)
        r, nrows, rp = _rows_arg(rows, M)
        Y = np.empty((N, nrows), dtype=np.float64)
        self._f("linear_codes")(_p(codes), _p(sc), _p(Xb), M, N, K, rp, nrows, _p(Y))
        return Y

    def linear(self, packed: np.ndarray, scales: np.ndarray, X: np.ndarray, M: int, K: int, rows=None) -> np.ndarray:
        _check_shape(M, K)
        packed = np.ascontiguousarray(packed, dtype=np.uint8)
        assert packed.size == self.packed_bytes(M, K)
        Xb = _u16(X)
        N, K2 = Xb.shape
        assert K2 == K
        sc = _u16(scales)
        assert sc.size == M
        r, nrows, rp = _rows_arg(rows, M)
        Y = np.empty((N, nrows), dtype=np.float64)
        if self._f("linear")(_p(packed), _p(sc), _p(Xb), M, N, K, rp, nrows, _p(Y)):
            raise MemoryError
        return Y

fp5 = NarrowOracle("fp5", 5, "e2m2")
fp4 = NarrowOracle("fp4", 4, "e2m1")
fp3 = NarrowOracle("fp3", 3, "e2m0")
BY_PREFIX = {"fp5": fp5, "fp4": fp4, "fp3": fp3}
