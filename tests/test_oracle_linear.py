"""Pins for the oracle's linear layer (CPU only): brute force, closed-form special cases,
linearity in K, and numpy's fp64 matmul of the unpacked matrix.
"""
import numpy as np

import workloads


def _setup(oracle, M, K, N, seed=0):
    W = workloads.make_weights(M, K, seed).numpy()
    X = workloads.make_activations(N, K, seed).numpy()
    packed, scales = oracle.quantize_pack(W)
    return W, X, packed, scales


def test_brute_force_tiny(oracle):
    M, K, N = 16, 256, 3
    W, X, packed, scales = _setup(oracle, M, K, N, seed=5)
    codes = oracle.unpack_codes(packed, M, K)
    table = [oracle.decode(c) for c in range(64)]
    Y = oracle.linear(packed, scales, X, M, K)
    assert Y.shape == (N, M)
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                acc += table[codes[m, k]] * float(X[n, k])
            assert Y[n, m] == float(scales[m]) * acc, (m, n)


def test_matches_numpy_matmul(oracle):
    name, M, K = workloads.TINY
    N = 8
    W, X, packed, scales = _setup(oracle, M, K, N)
    codes = oracle.unpack_codes(packed, M, K)
    Wd = oracle.decode_table()[codes] * scales.astype(np.float64)[:, None]
    ref = X.astype(np.float64) @ Wd.T                 # [N][M]
    Y = oracle.linear(packed, scales, X, M, K)
    scale = np.abs(ref).max()
    assert np.abs(Y - ref).max() <= 1e-12 * scale
    # the codes-based entry point agrees exactly with the packed one
    assert np.array_equal(oracle.linear_codes(codes, scales, X), Y)
    # and quantisation did something sensible: the fp16 GEMM of the original weights is close but not equal
    ref16 = X.astype(np.float64) @ W.astype(np.float64).T
    rel = np.abs(ref - ref16).max() / np.abs(ref16).max()
    assert 1e-4 < rel < 0.2


def test_all_ones_gives_column_sums(oracle):
    M, K, N = 32, 512, 5
    codes = np.full((M, K), 0b001100, dtype=np.uint8)          # every weight is 1.0
    scales = np.ones(M, dtype=np.float16)
    X = workloads.make_activations(N, K, 3).numpy()
    Y = oracle.linear(oracle.pack(codes), scales, X, M, K)
    sums = np.array([sum(float(v) for v in X[n]) for n in range(N)])    # sequential fp64 sums
    assert np.array_equal(Y, np.repeat(sums[:, None], M, axis=1))


def test_permutation_like_weights(oracle):
    """One non-zero 0.875 = 28 * 2^-5 per row: scale = 2^-5 exactly, code 31, Y[n][m] = 0.875 * X[n][pi(m)]."""
    M, K, N = 48, 512, 4
    rng = np.random.default_rng(11)
    pi = rng.permutation(K)[:M]
    W = np.zeros((M, K), dtype=np.float16)
    sign = rng.choice([-1.0, 1.0], M)
    W[np.arange(M), pi] = (0.875 * sign).astype(np.float16)
    X = workloads.make_activations(N, K, 4).numpy()
    packed, scales = oracle.quantize_pack(W)
    assert np.all(scales.astype(np.float64) == 2.0 ** -5)
    Y = oracle.linear(packed, scales, X, M, K)
    want = 0.875 * sign[None, :] * X.astype(np.float64)[:, pi]
    assert np.array_equal(Y, want)


def test_k_linearity_and_row_subsets(oracle):
    M, K, N = 32, 768, 4
    W, X, packed, scales = _setup(oracle, M, K, N, seed=9)
    codes = oracle.unpack_codes(packed, M, K)
    Y = oracle.linear_codes(codes, scales, X)
    K1 = 256
    Y1 = oracle.linear_codes(codes[:, :K1].copy(), scales, X[:, :K1].copy())
    Y2 = oracle.linear_codes(codes[:, K1:].copy(), scales, X[:, K1:].copy())
    assert np.abs(Y - (Y1 + Y2)).max() <= 1e-13 * np.abs(Y).max()
    rows = np.array([31, 0, 17, 5], dtype=np.int64)
    Ys = oracle.linear(packed, scales, X, M, K, rows=rows)
    assert Ys.shape == (N, 4)
    assert np.array_equal(Ys, Y[:, rows])
    # a transposed operand or a dropped scale would fail these
    assert not np.allclose(Y, oracle.linear_codes(codes, np.ones(M, dtype=np.float16), X))


def test_fp16_weight_linear(oracle):
    M, K, N = 32, 512, 3
    W = workloads.make_weights(M, K, 1).numpy()
    X = workloads.make_activations(N, K, 1).numpy()
    Y = oracle.linear_f16(W, X)
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    assert np.abs(Y - ref).max() <= 1e-12 * np.abs(ref).max()
