"""Pins for the 5-bit (e2m2) part of the oracle (CPU only).

Same kinds of pins as for e3m2: hand-evaluated values of the paper's Eq. 1 (tests/golden/), the bit-copy
cast of Section 5.3, Eq. 3 as an independent decode route, hand-derived ties, the quantizer's three exact
routes, the layout as a bijection and as a register-level reconstruction written from its description, and
the linear layer against brute force, closed forms and numpy's fp64 matmul.
"""
import os

import numpy as np
import pytest

import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def o5():
    from oracle import fpx_oracle
    return fpx_oracle.fp5


def _read(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            rows.append([float(t) for t in line.split()])
    return rows


def test_decode_matches_hand_table(o5):
    vals = [v for row in _read("e2m2_values.txt") for v in row]
    assert len(vals) == 16
    for c in range(16):
        assert o5.decode(c) == vals[c]
        assert o5.decode(c + 16) == -vals[c]
    assert np.signbit(o5.decode(16)) and o5.decode(16) == 0.0
    t = o5.decode_table()
    assert t[:16].sum() == 40.0 and t[:16].max() == 7.0
    assert np.all(np.diff(t[:16]) > 0)
    assert np.all(t * 4 == np.round(t * 4))


def test_decode_equals_bitcopy_cast(o5):
    """Section 5.3, Eq. 3 for e2m2: sign to bit 15, EEMM to bits 11..8 of an fp16 (E16 := Ex), times 2^(15-1)."""
    for c in range(32):
        bits = np.array([((c & 0x10) << 11) | ((c & 0x0F) << 8)], dtype=np.uint16)
        v = float(bits.view(np.float16)[0]) * 16384.0
        assert v == o5.decode(c), c
        assert np.signbit(v) == np.signbit(o5.decode(c))


def test_hand_ties(o5):
    one = int(np.array([1.0], dtype=np.float16).view(np.uint16)[0])
    for value, grid, g in _read("quantize_ties_e2m2.txt"):
        w = np.array([value], dtype=np.float16)
        assert float(w[0]) == value or abs(float(w[0]) - value) < 1e-3     # inputs are (near) fp16 values
        code = o5.quantize_one(int(w.view(np.uint16)[0]), one)
        assert code == int(g), (value, code)
        assert o5.decode(code) == grid
        assert o5.quantize_one(int((-w).view(np.uint16)[0]), one) == int(g) + 16


def test_scale_is_exactly_rounded_and_quantizer_routes_agree(o5):
    rng = np.random.default_rng(5)
    amax = rng.integers(1, 0x7C00, size=4000).astype(np.uint16)
    for a in amax[:2000]:
        a_val = float(np.array([a], dtype=np.uint16).view(np.float16)[0])
        want = np.float16(np.float64(a_val) / 7.0)        # fp64 quotient then one rounding: no double-rounding case
        assert o5.scale_for_amax(int(a)) == int(np.array([want]).view(np.uint16)[0])
    # three exact routes to the code: oracle (argmin of exact differences), fp32 divide + round to grid, midpoints
    table = o5.decode_table()[:16]
    mids = (table[1:] + table[:-1]) / 2
    W = workloads.make_weights(16, 256, seed=3).numpy()
    codes, scales = o5.quantize(W)
    for m in range(16):
        s = np.float64(scales[m])
        ratio = np.abs(W[m].astype(np.float64)) / s
        g = np.searchsorted(mids, ratio, side="left")      # ratio == mid goes to the lower index ...
        tie = np.isin(ratio, mids)
        g = np.where(tie & (g % 2 == 1), g + 1, g)         # ... unless the upper code is the even one
        g = np.minimum(g, 15)
        want = g + 16 * np.signbit(W[m]).astype(np.int64)
        assert np.array_equal(codes[m], want)


def test_every_code_round_trips(o5):
    for s in (2.0 ** -6, 0.01171875):
        row = np.array([o5.decode(c) * s for c in range(32)] * 8, dtype=np.float64)
        W = np.tile(row.astype(np.float16), (16, 1))
        assert np.all(W.astype(np.float64) == row)         # exact in fp16
        codes, scales = o5.quantize(W)
        assert np.all(scales.astype(np.float64) == s)
        assert np.array_equal(codes[0], np.tile(np.arange(32, dtype=np.uint8), 8))
        packed = o5.pack(codes)
        assert np.array_equal(o5.unpack_codes(packed, 16, 256), codes)
        Wd = o5.unpack(packed, scales, 16, 256)
        assert np.array_equal(Wd.view(np.uint16), W.view(np.uint16))      # -0 keeps its sign


def test_pos_is_a_bijection(o5):
    for M, K in ((16, 256), (32, 512)):
        seen = np.zeros(5 * M * K, dtype=np.uint8)
        for m in range(M):
            for k in range(K):
                for b in range(5):
                    p = o5.pos(M, K, m, k, b)
                    assert 0 <= p < 5 * M * K
                    seen[p] += 1
                    assert p // (2560 * 8) == (k // 256) * (M // 16) + m // 16
        assert np.all(seen == 1)
        assert o5.packed_bytes(M, K) == 5 * M * K // 8


def _swar_unpack_tile(tile_bytes):
    """One tile (2560 bytes) -> codes [16][256], rebuilt with whole-word shifts and masks as a lane would:
    five masked words give twenty codes in place, three three-term stitches give the other twelve.  Written
    from the layout's description, without pos()."""
    p01 = tile_bytes[:2048].view(np.uint32).reshape(2, 64, 4)
    p2 = tile_bytes[2048:].view(np.uint32).reshape(64, 2)
    codes = np.zeros((16, 256), dtype=np.uint8)
    for slot in range(64):
        r, q = slot % 16, slot // 16
        words = [int(p01[0][slot, i]) for i in range(4)] + [int(p01[1][slot, i]) for i in range(4)] + [int(p2[slot, 0]), int(p2[slot, 1])]
        for half in range(2):
            D = words[5 * half:5 * half + 5]
            B = [d & 0x8F8F8F8F for d in D]
            B.append(((D[0] << 1) & 0x80808080) | ((D[0] >> 2) & 0x0C0C0C0C) | ((D[1] >> 5) & 0x03030303))
            B.append(((D[1] << 3) & 0x80808080) | ((D[2] >> 3) & 0x0E0E0E0E) | ((D[3] >> 6) & 0x01010101))
            B.append(((D[3] << 2) & 0x80808080) | ((D[3] >> 1) & 0x08080808) | ((D[4] >> 4) & 0x07070707))
            for w in range(8):
                for byte in range(4):
                    v = (B[w] >> (8 * byte)) & 0xFF
                    assert v & 0x70 == 0
                    i = 4 * w + byte
                    run, j = 4 * half + i // 8, i % 8
                    codes[r, run * 32 + q * 8 + j] = ((v >> 7) << 4) | (v & 0x0F)
    return codes


def test_register_level_reconstruction(o5):
    M, K = 32, 512
    codes = (workloads.make_codes(M, K, 9).numpy() & 31).astype(np.uint8)
    packed = o5.pack(codes)
    tiles = packed.reshape(K // 256, M // 16, 2560)
    for rt in range(M // 16):
        for kt in range(K // 256):
            got = _swar_unpack_tile(tiles[kt, rt])
            assert np.array_equal(got, codes[rt * 16:(rt + 1) * 16, kt * 256:(kt + 1) * 256])
    assert np.array_equal(o5.unpack_codes(packed, M, K), codes)


def test_unpack_is_layout_independent(o5):
    name, M, K = workloads.TINY
    W = workloads.make_weights(M, K, seed=0).numpy()
    codes, scales = o5.quantize(W)
    packed, scales2 = o5.quantize_pack(W)
    assert np.array_equal(scales.view(np.uint16), scales2.view(np.uint16))
    want = (o5.decode_table()[codes] * scales.astype(np.float64)[:, None]).astype(np.float16)
    got = o5.unpack(packed, scales2, M, K)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
    # every row reaches a +-7 code; the error is at most half a step of the top binade (0.5 * scale), plus the
    # rounding of the scale (the row maximum may sit 7 * 2^-11 * scale above the grid) and of the fp16 result
    assert np.all((codes & 15).max(axis=1) == 15)
    err = np.abs(got.astype(np.float64) - W.astype(np.float64))
    assert np.all(err <= (0.5 + 7 * 2.0 ** -10) * scales.astype(np.float64)[:, None])


def test_linear_against_brute_force_and_numpy(o5):
    M, K, N = 32, 512, 5
    W = workloads.make_weights(M, K, seed=4).numpy()
    X = workloads.make_activations(N, K, seed=4).numpy()
    packed, scales = o5.quantize_pack(W)
    codes = o5.unpack_codes(packed, M, K)
    Y = o5.linear(packed, scales, X, M, K)
    table = o5.decode_table()
    Wd = table[codes] * scales.astype(np.float64)[:, None]
    brute = np.zeros((N, M))
    for n in range(N):
        for m in range(0, M, 7):
            acc = 0.0
            for k in range(K):
                acc += table[codes[m, k]] * float(X[n, k])
            brute[n, m] = float(scales[m]) * acc
    assert np.allclose(Y[:, ::7], brute[:, ::7], rtol=1e-13, atol=0)
    assert np.allclose(Y, X.astype(np.float64) @ Wd.T, rtol=1e-11, atol=1e-12)
    rows = np.array([3, 17, 31])
    assert np.array_equal(o5.linear(packed, scales, X, M, K, rows=rows), Y[:, rows])


def test_linear_closed_forms(o5):
    M, K, N = 16, 256, 3
    X = workloads.make_activations(N, K, seed=1).numpy()
    # all codes = 0b00100 (1.0), scale 1: column sums of X
    codes = np.full((M, K), 0b00100, dtype=np.uint8)
    ones = np.ones(M, dtype=np.float16)
    Y = o5.linear(o5.pack(codes), ones, X, M, K)
    assert np.allclose(Y, X.astype(np.float64).sum(axis=1)[:, None], rtol=1e-13)
    # one non-zero 0.875 = 7 * 2^-3 per row at column pi(m): scale 2^-3, code 15, Y = 0.875 * X[pi(m)]
    W = np.zeros((M, K), dtype=np.float16)
    pi = (np.arange(M) * 37 + 5) % K
    W[np.arange(M), pi] = 0.875
    packed, scales = o5.quantize_pack(W)
    assert np.all(scales.astype(np.float64) == 0.125)
    Y = o5.linear(packed, scales, X, M, K)
    assert np.array_equal(Y, 0.875 * X.astype(np.float64)[:, pi])
