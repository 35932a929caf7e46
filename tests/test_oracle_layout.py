"""Pins for the oracle's packed layout (CPU only): the bit map is a bijection with no padding,
pack/unpack round-trips, and the word-level shift/mask reconstruction that the
kernels use (restated here in numpy, from the layout's description) recovers the codes.
"""
import numpy as np

import workloads


def _all_pos(oracle, M, K):
    out = np.empty((M, K, 6), dtype=np.int64)
    for m in range(M):
        for k in range(K):
            for b in range(6):
                out[m, k, b] = oracle.pos(M, K, m, k, b)
    return out


def test_pos_is_a_bijection_smallest_tile(oracle):
    M, K = 16, 256
    p = _all_pos(oracle, M, K).ravel()
    assert p.min() == 0 and p.max() == 6 * M * K - 1
    assert np.unique(p).size == 6 * M * K


def test_pos_is_a_bijection_multi_tile(oracle):
    M, K = 48, 768           # 3 row tiles x 3 k tiles
    p = _all_pos(oracle, M, K).ravel()
    assert p.min() == 0 and p.max() == 6 * M * K - 1
    assert np.unique(p).size == 6 * M * K
    # tiles are k-tile major and 3072 bytes each: weight (m, k) lives in tile (k//256)*(M//16) + m//16
    for (m, k) in [(0, 0), (15, 255), (16, 0), (17, 300), (47, 767)]:
        tile = (k // 256) * (M // 16) + m // 16
        for b in range(6):
            assert oracle.pos(M, K, m, k, b) // (3072 * 8) == tile


def test_packed_size_and_no_padding(oracle):
    for (M, K) in [(16, 256), (256, 512), (8192, 22016)]:
        assert oracle.packed_bytes(M, K) == 3 * M * K // 4
    ones = np.full((32, 512), 63, dtype=np.uint8)
    assert np.all(oracle.pack(ones) == 0xFF)           # every bit of the stream belongs to a code
    assert np.all(oracle.pack(np.zeros((32, 512), dtype=np.uint8)) == 0)


def test_pack_unpack_round_trip(oracle):
    for (M, K, seed) in [(16, 256, 0), (256, 512, 1), (80, 1280, 2)]:
        codes = workloads.make_codes(M, K, seed).numpy()
        packed = oracle.pack(codes)
        assert packed.size == 3 * M * K // 4
        assert np.array_equal(oracle.unpack_codes(packed, M, K), codes)
    # single-bit probes: one code bit set -> exactly one stream bit set, at pos()
    M, K = 32, 512
    rng = np.random.default_rng(3)
    for _ in range(50):
        m, k, b = int(rng.integers(M)), int(rng.integers(K)), int(rng.integers(6))
        codes = np.zeros((M, K), dtype=np.uint8)
        codes[m, k] = 1 << b
        packed = oracle.pack(codes)
        bits = np.flatnonzero(np.unpackbits(packed, bitorder="little"))
        assert bits.tolist() == [oracle.pos(M, K, m, k, b)]


def _lane_stream_unpack_tile_words(words):
    """words: uint32 [3][64][4] of one tile (plane, slot, word).  Returns codes [16][256] rebuilt the way a
    lane of the kernels sees the tile: the slot's 12 words (plane-major) are two 192-bit little-endian
    streams of 32 six-bit fields, field i of stream c being column 8*(i%8... see below) - written from the
    layout's description, without pos()."""
    codes = np.zeros((16, 256), dtype=np.uint8)
    for slot in range(64):
        r, q = slot % 16, slot // 16
        lane_words = [int(words[p][slot, w]) for p in range(3) for w in range(4)]      # 12 words, plane-major
        for c in range(2):
            stream = 0
            for w in range(6):
                stream |= lane_words[6 * c + w] << (32 * w)
            for i in range(32):
                run, j = 4 * c + i // 8, i % 8
                codes[r, run * 32 + q * 8 + j] = (stream >> (6 * i)) & 0x3F
    return codes


def test_register_level_reconstruction(oracle):
    M, K = 32, 512
    codes = workloads.make_codes(M, K, 7).numpy()
    packed = oracle.pack(codes)
    tiles = packed.view(np.uint32).reshape(K // 256, M // 16, 3, 64, 4)
    for rt in range(M // 16):
        for kt in range(K // 256):
            got = _lane_stream_unpack_tile_words(tiles[kt, rt])
            assert np.array_equal(got, codes[rt * 16:(rt + 1) * 16, kt * 256:(kt + 1) * 256])


def test_unpack_is_layout_independent(oracle):
    """unpack(quantize_pack(W)) == decode(quantize(W)) * scale rounded once to fp16, computed
    row-major with numpy without touching pos()."""
    name, M, K = workloads.TINY
    W = workloads.make_weights(M, K, seed=0).numpy()
    codes, scales = oracle.quantize(W)
    packed, scales2 = oracle.quantize_pack(W)
    assert np.array_equal(scales.view(np.uint16), scales2.view(np.uint16))
    table = oracle.decode_table()
    want = (table[codes] * scales.astype(np.float64)[:, None]).astype(np.float16)   # exact product, one rounding
    got = oracle.unpack(packed, scales2, M, K)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
    # quantisation error is bounded by half a grid step of the top binade: |W - Wd| <= 2 * scale
    # (plus the single fp16 rounding of the dequantised value)
    gd = got.astype(np.float64)
    assert np.all(np.abs(gd - W.astype(np.float64)) <= 2.0 * scales.astype(np.float64)[:, None] + 2.0 ** -11 * np.abs(gd))
