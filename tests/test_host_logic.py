"""CPU checks of arithmetic shortcuts that the HIP kernels take, restated in numpy from their description
and compared with the oracle's exact definition over many more cases than a GPU test can afford.

The quantizer kernel does not divide: it multiplies by a reciprocal, applies one fused-remainder correction
and rounds the fp32 quotient onto the e3m2 grid with integer bit tricks.  That this equals the exact
round-to-nearest-even of |w|/scale (ties included) is an argument about fp32 arithmetic; here it is tested.
"""
import numpy as np


def _gpu_style_codes(w_bits: np.ndarray, s_bits: np.ndarray) -> np.ndarray:
    """w_bits, s_bits: uint16 arrays (broadcastable).  Emulates the kernel's steps in fp32 (fma via fp64)."""
    w_bits, s_bits = np.broadcast_arrays(w_bits, s_bits)
    sign = (w_bits >> 15).astype(np.uint32)
    a = (w_bits & 0x7FFF).astype(np.uint16).view(np.float16).astype(np.float32)
    s = (s_bits & 0x7FFF).astype(np.uint16).view(np.float16).astype(np.float32)
    with np.errstate(divide="ignore"):
        inv = np.where(s == 0, np.float32(0), (np.float32(1) / s)).astype(np.float32)
    q = (a * inv).astype(np.float32)
    rem = (a.astype(np.float64) - q.astype(np.float64) * s.astype(np.float64)).astype(np.float32)   # fma(-q, s, a)
    ratio = (rem.astype(np.float64) * inv.astype(np.float64) + q.astype(np.float64)).astype(np.float32)  # fma(rem, inv, q)
    small = np.where(ratio < np.float32(0.25), ratio, np.float32(0))        # the other lanes take the normal route
    sub = np.rint(small * np.float32(16)).astype(np.uint32)                 # ratio < 0.25: multiples of 1/16
    u = ratio.view(np.uint32).astype(np.uint64)
    u = u + 0x000FFFFF + ((u >> 21) & 1)
    nor = ((u >> 21) - (124 << 2)).astype(np.int64)
    g = np.where(ratio < np.float32(0.25), sub.astype(np.int64), nor)
    g = np.minimum(g, 31).astype(np.uint32)
    return (sign << 5) | g


def _oracle_codes(oracle, w_bits, s_bits):
    w_bits, s_bits = np.broadcast_arrays(w_bits, s_bits)
    out = np.empty(w_bits.shape, dtype=np.uint32)
    it = np.nditer([w_bits, s_bits, out], op_flags=[["readonly"], ["readonly"], ["writeonly"]])
    for w, s, o in it:
        o[...] = oracle.quantize_one(int(w), int(s))
    return out


def test_quantizer_shortcut_random(oracle):
    rng = np.random.default_rng(0)
    s_bits = np.concatenate([rng.integers(1, 0x7BFF, 300), rng.integers(0x1800, 0x2400, 300), [0, 1, 2, 0x3FF, 0x400, 0x3C00]]).astype(np.uint16)
    w_bits = rng.integers(0, 0x10000, (s_bits.size, 60)).astype(np.uint16)
    w_bits = np.where((w_bits & 0x7C00) == 0x7C00, np.uint16(0x1234), w_bits)     # finite only
    got = _gpu_style_codes(w_bits, s_bits[:, None])
    want = _oracle_codes(oracle, w_bits, s_bits[:, None])
    assert np.array_equal(got, want)


def test_quantizer_shortcut_on_exact_ties(oracle):
    """Every (scale, midpoint) pair whose product is an fp16: |w| = midpoint * scale exactly."""
    grid = oracle.decode_table()[:32]
    mids = (grid[:-1] + grid[1:]) / 2
    s_bits = np.arange(1, 0x7BFF, 7, dtype=np.uint16)
    s = s_bits.view(np.float16).astype(np.float64)
    with np.errstate(over="ignore"):
        prod = mids[None, :] * s[:, None]
    with np.errstate(over="ignore"):
        h = prod.astype(np.float16)
    exact = (h.astype(np.float64) == prod) & np.isfinite(h.astype(np.float64))
    rows, cols = np.nonzero(exact)
    assert rows.size > 10000
    w_bits = h.view(np.uint16)[rows, cols]
    sb = s_bits[rows]
    got = _gpu_style_codes(w_bits, sb)
    # ties go to the even code: midpoint j sits between codes j and j+1
    want = np.where(cols % 2 == 0, cols, cols + 1).astype(np.uint32)
    assert np.array_equal(got, want)
    # neighbours of the ties (one fp16 ulp either side) against the oracle, on a sample
    idx = np.random.default_rng(1).choice(rows.size, 3000, replace=False)
    for d in (-1, 1):
        wb = (w_bits[idx].astype(np.int32) + d).clip(0, 0x7BFF).astype(np.uint16)
        assert np.array_equal(_gpu_style_codes(wb, sb[idx]), _oracle_codes(oracle, wb, sb[idx]))
    # and the oracle agrees on the ties themselves (sample)
    assert np.array_equal(_oracle_codes(oracle, w_bits[idx], sb[idx]), want[idx])
