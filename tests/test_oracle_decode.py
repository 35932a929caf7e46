"""Pins for the oracle's e3m2 decode and its fp16 conversions (CPU only).

The decode is pinned to (a) hand-evaluated values of the paper's Eq. 1 stored in
tests/golden/, (b) the bit-copy cast of Section 5.3, Eq. 3, evaluated with numpy's
float16 (a second, independent route), (c) the byte-wise mask sequence of
Algorithm 1 (a third route), and (d) structural facts of the format.
"""
import os
from fractions import Fraction

import numpy as np

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_values():
    vals = []
    with open(os.path.join(GOLDEN, "e3m2_values.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            vals += [float(t) for t in line.split()]
    assert len(vals) == 32
    return vals


def test_decode_matches_hand_table(oracle):
    vals = _golden_values()
    for c in range(32):
        assert oracle.decode(c) == vals[c], c
        assert oracle.decode(c + 32) == -vals[c], c
    # the sign of code 32 is a negative zero
    assert np.signbit(oracle.decode(32)) and oracle.decode(32) == 0.0
    assert not np.signbit(oracle.decode(0))


def test_named_codes(oracle):
    # the benchmark spec's example and three more hand values
    assert oracle.decode(0b011111) == 28.0
    assert oracle.decode(0b000001) == 1.0 / 16
    assert oracle.decode(0b000100) == 0.25
    assert oracle.decode(0b001100) == 1.0
    assert oracle.decode(0b111111) == -28.0


def test_structure(oracle):
    t = oracle.decode_table()
    pos = t[:32]
    assert pos.sum() == 175.0
    assert np.all(np.diff(pos) > 0)                      # strictly increasing in the magnitude code
    assert np.all(pos * 16 == np.round(pos * 16))        # multiples of 1/16
    assert pos.max() == 28.0 and pos[1] == 0.0625
    assert np.all(t.astype(np.float16).astype(np.float64) == t)   # exact in fp16
    # three significant bits at most: value = integer <= 7 times a power of two
    for v in pos[1:]:
        fr = Fraction(float(v))
        num = fr.numerator
        while num % 2 == 0:
            num //= 2
        assert num <= 7


def test_decode_equals_bitcopy_cast(oracle):
    """Section 5.3, Eq. 3: copy sign and EEEMM into an fp16 (E16 := Ex), multiply by 2^(15-3)."""
    for c in range(64):
        bits = np.array([((c & 0x20) << 10) | ((c & 0x1F) << 8)], dtype=np.uint16)
        v = float(bits.view(np.float16)[0]) * 4096.0
        assert v == oracle.decode(c), c
        assert np.signbit(v) == np.signbit(oracle.decode(c))


def test_decode_equals_word_parallel_cast(oracle):
    """Section 5.3 casts several codes per 32-bit operation.  Derived here from the field positions alone:
    a code s|EEE|MM stored in the top six bits of a byte (bit 7 = s, bits 6..2 = EEEMM) becomes the high byte
    of an fp16 when s stays at bit 7 and EEEMM moves down to bits 4..0 - the fp16 pattern s 00EEE MM 00000000
    of Eq. 3.  On a word of four such bytes that is one mask for the four signs (bit 7 of every byte), one
    shift-and-mask for the four five-bit fields (field width 5 -> 0x1f per byte), and an OR; a byte at an odd
    position of the word is already the high byte of a half, a byte at an even position has to move up by 8."""
    SIGNS = sum(0x80 << (8 * i) for i in range(4))
    FIELDS = sum(0x1F << (8 * i) for i in range(4))
    ODD_BYTES = 0xFF00FF00
    rng = np.random.default_rng(0)
    for _ in range(64):
        codes = [int(c) for c in rng.integers(0, 64, size=4)]
        word = sum((c << 2) << (8 * i) for i, c in enumerate(codes))      # byte i = code i in the top six bits
        high_bytes = (word & SIGNS) | ((word >> 2) & FIELDS)               # every byte: s 00 EEEMM
        pair_odd = high_bytes & ODD_BYTES                                  # halves [byte1 00], [byte3 00]
        pair_even = (high_bytes << 8) & ODD_BYTES                          # halves [byte0 00], [byte2 00]
        got = {0: pair_even & 0xFFFF, 2: pair_even >> 16, 1: pair_odd & 0xFFFF, 3: pair_odd >> 16}
        for i, c in enumerate(codes):
            h = np.array([got[i]], dtype=np.uint16).view(np.float16)[0]
            assert float(h) * 4096.0 == oracle.decode(c), (i, c)


def test_half_to_double_exhaustive(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    for b in range(65536):
        v = oracle.half_to_double(b)
        if np.isnan(ref[b]):
            assert np.isnan(v)
        else:
            assert v == ref[b] and np.signbit(v) == np.signbit(ref[b]), b


def test_double_to_half_against_numpy(oracle):
    rng = np.random.default_rng(1)
    xs = []
    # random magnitudes over the whole fp16 range, including the subnormal range and overflow
    xs += list(np.ldexp(rng.uniform(0.5, 1.0, 4000), rng.integers(-30, 18, 4000)) * rng.choice([-1, 1], 4000))
    # every midpoint between adjacent fp16 values (the tie cases) and its two neighbours in double
    allh = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mids = (allh[:-1] + allh[1:]) / 2
    xs += list(mids[::7]) + list(np.nextafter(mids[::7], np.inf)) + list(np.nextafter(mids[::7], -np.inf))
    xs += [0.0, -0.0, 65504.0, 65519.99, 65520.0, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0000001]
    for x in xs:
        with np.errstate(over="ignore"):
            ref = int(np.array([x], dtype=np.float64).astype(np.float16).view(np.uint16)[0])
        assert oracle.double_to_half(float(x)) == ref, x
