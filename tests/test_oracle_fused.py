"""Pins for the oracle's linear layer with the decoder block's element-wise steps attached
(bias, silu(gate) * up, residual; Section 7.3's models) - CPU only.

The plain product is pinned elsewhere (test_oracle_linear.py); here each added step is pinned by
what fixes it: the identity case, additivity with distinct per-row / per-element addends (an index
or transposition mistake moves them), textbook values of the logistic function through
scipy.special.expit on products crafted to be exact, and the order of the three steps.
"""
import numpy as np
import pytest
from scipy.special import expit

import workloads

CODE_ONE = 0b001100   # e3m2: E = 3, M = 0 -> 1.0
CODE_TWO = 0b010000   # E = 4 -> 2.0


def _setup(oracle, M, K, N, seed=0):
    W = workloads.make_weights(M, K, seed).numpy()
    X = workloads.make_activations(N, K, seed).numpy()
    packed, scales = oracle.quantize_pack(W)
    return X, packed, scales


def test_no_step_is_the_plain_layer(oracle):
    M, K, N = 32, 512, 5
    X, packed, scales = _setup(oracle, M, K, N, seed=3)
    assert np.array_equal(oracle.linear_fused(packed, scales, X, M, K), oracle.linear(packed, scales, X, M, K))


def test_bias_is_added_per_output_row(oracle):
    M, K, N = 32, 256, 4
    X, packed, scales = _setup(oracle, M, K, N, seed=4)
    bias = (np.arange(M) * 0.25 - 3.0).astype(np.float16)          # distinct, exact in fp16
    plain = oracle.linear(packed, scales, X, M, K)
    got = oracle.linear_fused(packed, scales, X, M, K, bias=bias)
    assert np.abs((got - plain) - bias.astype(np.float64)[None, :]).max() <= 1e-12 * np.abs(plain).max()


def test_residual_is_added_per_element(oracle):
    M, K, N = 32, 256, 4
    X, packed, scales = _setup(oracle, M, K, N, seed=5)
    R = (np.arange(N * M).reshape(N, M) * 0.125 - 7.0).astype(np.float16)   # R[n][m] all distinct
    plain = oracle.linear(packed, scales, X, M, K)
    got = oracle.linear_fused(packed, scales, X, M, K, residual=R)
    assert np.abs((got - plain) - R.astype(np.float64)).max() <= 1e-12 * np.abs(plain).max()


def _crafted(oracle, gates, ups, K=256):
    """16 weight rows = 8 (gate, up) pairs; pair i has gate row = 1.0 at column 2i and up row = 2.0 at
    column 2i+1 (scale 1), so with X[n][2i] = gates[n][i] and X[n][2i+1] = ups[n][i] / 2 the two
    products are exactly gates and ups."""
    M = 16
    codes = np.zeros((M, K), dtype=np.uint8)
    for i in range(8):
        codes[2 * i, 2 * i] = CODE_ONE
        codes[2 * i + 1, 2 * i + 1] = CODE_TWO
    packed = oracle.pack(codes)
    scales = np.ones(M, dtype=np.float16)
    N = gates.shape[0]
    X = np.zeros((N, K), dtype=np.float16)
    X[:, 0:16:2] = gates
    X[:, 1:16:2] = ups / 2
    return packed, scales, X, M, K


def test_gate_values_against_the_logistic_function(oracle):
    gates = np.array([[0.0, 1.0, -1.0, 2.0, -2.0, 20.0, -20.0, 0.5]], dtype=np.float16)
    ups = np.array([[3.0, 3.0, 3.0, -1.5, 5.0, 1.0, 1.0, 0.25]], dtype=np.float16)
    packed, scales, X, M, K = _crafted(oracle, gates, ups)
    got = oracle.linear_fused(packed, scales, X, M, K, gated=True)
    assert got.shape == (1, 8)
    g, u = gates.astype(np.float64), ups.astype(np.float64)
    want = g * expit(g) * u
    assert np.abs(got - want).max() <= 1e-14 * np.abs(want).max()
    # textbook anchors: silu(0) = 0, silu(1) = 1/(1 + 1/e), silu(x) - silu(-x) = x
    assert got[0, 0] == 0.0
    assert abs(got[0, 1] / 3.0 - 0.7310585786300049) < 1e-15
    assert abs(got[0, 1] / 3.0 - got[0, 2] / 3.0 - 1.0) < 1e-15
    # even row is the gate, odd row the value: the other way round would give silu(3) * 1
    assert abs(got[0, 1] - 3.0 * 0.7310585786300049) < 1e-14


def test_order_bias_then_gate_then_residual(oracle):
    gates = np.array([[1.0] * 8, [-0.5] * 8], dtype=np.float16)
    ups = np.array([[2.0] * 8, [4.0] * 8], dtype=np.float16)
    packed, scales, X, M, K = _crafted(oracle, gates, ups)
    bias = np.zeros(M, dtype=np.float16)
    bias[0::2] = np.arange(8) * 0.5        # shifts the gate of pair i
    bias[1::2] = -np.arange(8) * 0.25      # shifts the value of pair i
    R = (np.arange(16).reshape(2, 8) - 4.0).astype(np.float16)
    got = oracle.linear_fused(packed, scales, X, M, K, bias=bias, residual=R, gated=True)
    g = gates.astype(np.float64) + bias[0::2].astype(np.float64)[None, :]
    u = ups.astype(np.float64) + bias[1::2].astype(np.float64)[None, :]
    want = g * expit(g) * u + R.astype(np.float64)
    assert np.abs(got - want).max() <= 1e-14 * np.abs(want).max()


def test_listed_rows_are_output_rows(oracle):
    M, K, N = 64, 256, 3
    X, packed, scales = _setup(oracle, M, K, N, seed=6)
    bias = workloads.make_activations(1, M, 9).numpy()[0]
    R = workloads.make_activations(N, M // 2, 10).numpy()
    full = oracle.linear_fused(packed, scales, X, M, K, bias=bias, residual=R, gated=True)
    rows = np.array([31, 0, 7, 16], dtype=np.int64)
    part = oracle.linear_fused(packed, scales, X, M, K, bias=bias, residual=R, gated=True, rows=rows)
    assert np.array_equal(part, full[:, rows])
    rows = np.array([63, 2], dtype=np.int64)
    R2 = workloads.make_activations(N, M, 11).numpy()
    full = oracle.linear_fused(packed, scales, X, M, K, bias=bias, residual=R2)
    assert np.array_equal(oracle.linear_fused(packed, scales, X, M, K, bias=bias, residual=R2, rows=rows), full[:, rows])


def test_gated_needs_even_rows_and_matching_shapes(oracle):
    M, K, N = 16, 256, 2
    X, packed, scales = _setup(oracle, M, K, N)
    with pytest.raises(AssertionError):
        oracle.linear_fused(packed, scales, X, M, K, residual=np.zeros((N, M), np.float16), gated=True)


@pytest.mark.parametrize("bits", [5, 4, 3])
def test_other_widths_share_the_steps(oracle, bits):
    """The steps are one piece of code for every width (bits = 6 is the function pinned above); what changes
    is the linear layer under them, each pinned in its own file: with no step the result is that layer, and
    with all steps it is that layer's output pushed through the logistic function of scipy."""
    import importlib
    from oracle import fpx_oracle
    o = fpx_oracle.BY_PREFIX["fp%d" % bits]
    M, K, N = 32, 512, 3
    W = workloads.make_weights(M, K, seed=bits).numpy()
    X = workloads.make_activations(N, K, seed=bits).numpy()
    packed, scales = o.quantize_pack(W)
    Z = o.linear(packed, scales, X, M, K)
    assert np.array_equal(oracle.linear_fused(packed, scales, X, M, K, bits=bits), Z)
    bias = (workloads.make_activations(1, M, 40)[0] * 0.5).to(dtype=workloads.make_weights(1, 1).dtype).numpy()
    R = workloads.make_activations(N, M // 2, 41).numpy()
    got = oracle.linear_fused(packed, scales, X, M, K, bias=bias, residual=R, gated=True, bits=bits)
    z = Z + bias.astype(np.float64)[None, :]
    want = z[:, 0::2] * expit(z[:, 0::2]) * z[:, 1::2] + R.astype(np.float64)
    assert np.abs(got - want).max() <= 1e-13 * np.abs(want).max()


def test_group_scales_share_the_steps(oracle):
    from oracle import fp6g_oracle
    M, K, N = 32, 512, 3
    W = workloads.make_weights(M, K, seed=12).numpy()
    X = workloads.make_activations(N, K, seed=12).numpy()
    packed, scales = fp6g_oracle.quantize_pack(W, 128)
    Z = fp6g_oracle.linear(packed, scales, X, M, K, 128)
    assert np.array_equal(oracle.linear_fused(packed, scales, X, M, K, group=128), Z)
    R = workloads.make_activations(N, M, 42).numpy()
    got = oracle.linear_fused(packed, scales, X, M, K, residual=R, group=128)
    assert np.abs(got - (Z + R.astype(np.float64))).max() <= 1e-13 * np.abs(Z).max()
