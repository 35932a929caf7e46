"""Pins for the group-wise-scale part of the oracle (CPU only): it must reduce to the per-row oracle, which
is pinned on its own, in every way the definition allows."""
import numpy as np
import pytest

import workloads


@pytest.fixture(scope="module")
def og():
    from oracle import fp6g_oracle
    return fp6g_oracle


def test_one_group_per_row_is_the_per_row_scheme(og, oracle):
    M, K = 32, 512
    W = workloads.make_weights(M, K, seed=2).numpy()
    codes_g, scales_g = og.quantize(W, K)
    codes_r, scales_r = oracle.quantize(W)
    assert np.array_equal(codes_g, codes_r)
    assert np.array_equal(scales_g[:, 0].view(np.uint16), scales_r.view(np.uint16))
    X = workloads.make_activations(3, K, seed=2).numpy()
    packed_g, sg = og.quantize_pack(W, K)
    packed_r, sr = oracle.quantize_pack(W)
    assert np.array_equal(packed_g, packed_r)
    assert np.allclose(og.linear(packed_g, sg, X, M, K, K), oracle.linear(packed_r, sr, X, M, K), rtol=1e-13, atol=0)
    assert np.array_equal(og.unpack(packed_g, sg, M, K, K).view(np.uint16), oracle.unpack(packed_r, sr, M, K).view(np.uint16))


@pytest.mark.parametrize("group", [128, 256])
def test_every_group_is_quantized_like_a_row_of_its_own(og, oracle, group):
    M, K = 16, 768
    W = workloads.make_weights(M, K, seed=3).numpy()
    W[3, 130:140] *= 8                       # groups of one row with very different ranges
    W[5, 0:256] = 0
    codes, scales = og.quantize(W, group)
    assert scales.shape == (M, K // group)
    for g in range(K // group):
        slab = np.ascontiguousarray(W[:, g * group:(g + 1) * group])
        c, s = oracle.quantize(slab)
        assert np.array_equal(codes[:, g * group:(g + 1) * group], c)
        assert np.array_equal(scales[:, g].view(np.uint16), s.view(np.uint16))
    assert np.all(scales[5, 0] == 0) and np.all((codes[5, :256] & 31) == 0)


def test_unpack_and_linear_are_sums_over_groups(og, oracle):
    M, K, N, group = 32, 512, 4, 128
    W = workloads.make_weights(M, K, seed=4).numpy()
    W[:, 128:256] *= 3
    X = workloads.make_activations(N, K, seed=4).numpy()
    packed, scales = og.quantize_pack(W, group)
    codes = oracle.unpack_codes(packed, M, K)
    table = oracle.decode_table()
    Wd = table[codes] * np.repeat(scales.astype(np.float64), group, axis=1)           # exact products
    assert np.array_equal(og.unpack(packed, scales, M, K, group).view(np.uint16), Wd.astype(np.float16).view(np.uint16))
    Y = og.linear(packed, scales, X, M, K, group)
    assert np.allclose(Y, X.astype(np.float64) @ Wd.T, rtol=1e-11, atol=1e-12)
    # group by group with the pinned per-row routine
    total = np.zeros_like(Y)
    for g in range(K // group):
        sl = slice(g * group, (g + 1) * group)
        total += oracle.linear_codes(np.ascontiguousarray(codes[:, sl]), scales[:, g].copy(), np.ascontiguousarray(X[:, sl]))
    assert np.allclose(Y, total, rtol=1e-12, atol=1e-13)
    rows = np.array([1, 30])
    assert np.array_equal(og.linear(packed, scales, X, M, K, group, rows=rows), Y[:, rows])
    # finer scales never quantize worse than one scale per row
    Wd_row = oracle.unpack(*oracle.quantize_pack(W), M, K).astype(np.float64)
    assert np.abs(Wd - W.astype(np.float64)).sum() < np.abs(Wd_row - W.astype(np.float64)).sum()
