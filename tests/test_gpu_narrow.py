"""GPU parity tests of the 5-bit (e2m2), 4-bit (e2m1) and 3-bit (e2m0) calls, through the C-ABI binding,
against the CPU oracle, every test once per width.

pack / unpack bit for bit; the GEMM within max_m |Y_gpu - Y_ref| <= 5e-3 * max_m |Y_ref| per output column.
"""
import numpy as np
import pytest
import torch

import workloads
from gpu_checks import check_linear as _check_linear
from packed_rows import row_tiles_of

pytestmark = pytest.mark.gpu


class Width:
    """What differs between the widths: the calls, the largest magnitude, hand-picked ties, tile bytes."""

    def __init__(self, prefix, bits, top, ties, tile_bytes, unit, small, tile_cols=256):
        self.prefix, self.bits, self.top, self.ties, self.tile_bytes = prefix, bits, top, ties, tile_bytes
        self.tile_cols = tile_cols
        self.unit = unit      # a value v with v / top * top exact in fp16: one non-zero per row gives scale v / top
        self.small = small    # three small multiples of 2^-24 (row of a subnormal scale) and one whose scale rounds down
        self.codes = 1 << bits


WIDTHS = {
    "fp5": Width("fp5", 5, 7.0, [6.5, 5.5, 4.5, 3.75, 1.875, 0.875, 0.375, 0.125, 6.75, 2.2, 2.3, 0.13, 0.12], 2560, 0.875,
                 (7, 3, 2, 10)),
    "fp4": Width("fp4", 4, 6.0, [5, 3.5, 2.5, 1.75, 1.25, 0.75, 0.25, 5.5, 4.5, 2.4, 2.6, 0.26, 0.24], 2048, 0.75,
                 (6, 3, 2, 8)),
    "fp3": Width("fp3", 3, 4.0, [3, 1.5, 0.5, 3.1, 2.9, 3.5, 1.6, 1.4, 0.51, 0.49], 3072, 0.75, (4, 2, 1, 5), tile_cols=512),
}


@pytest.fixture(scope="module", params=sorted(WIDTHS))
def wd(request):
    return WIDTHS[request.param]


@pytest.fixture(scope="module")
def pkg():
    import paper_2401_14112_amd as p

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    p.load_library()
    return p


@pytest.fixture(scope="module")
def o5(wd):
    from oracle import fpx_oracle
    return fpx_oracle.BY_PREFIX[wd.prefix]


def _call(pkg, wd, name):
    return getattr(pkg, "%s_%s" % (wd.prefix, name))


def _say(msg):
    print(msg, flush=True)


def _np(t):
    return t.detach().cpu().numpy()


def _special_matrix(o5, wd):
    """Every code under several scales, hand ties, signed zeros, zero rows, subnormal scales, huge values."""
    table = o5.decode_table()
    M, K = 32, 512
    W = np.zeros((M, K), dtype=np.float16)
    for m, s in enumerate([2.0 ** -6, 0.01171875, 1.0, 3.0]):
        W[m, :wd.codes] = (table * s).astype(np.float16)
        W[m, 100:100 + wd.codes] = (table[::-1] * s).astype(np.float16)
    ties = wd.ties
    W[4, 0] = wd.top
    W[4, 1:1 + len(ties)] = ties
    W[5, 0] = -wd.top
    W[5, 1:1 + len(ties)] = [-t for t in ties]
    W[6, 3] = -0.0
    W[7, :] = np.float16(2.0 ** -24)                 # amax / top rounds to a zero scale
    W[7, 5] = -np.float16(2.0 ** -24)
    W[8, 0] = np.float16(wd.small[0] * 2.0 ** -24)   # subnormal scale 2^-24
    W[8, 1] = np.float16(wd.small[1] * 2.0 ** -24)
    W[8, 2] = -np.float16(wd.small[2] * 2.0 ** -24)
    W[9, 0] = np.float16(wd.small[3] * 2.0 ** -24)   # scale rounds down so the row maximum saturates
    W[9, 1] = np.float16(3 * 2.0 ** -24)
    W[10, :] = np.float16(65504.0)
    W[11, 7] = np.float16(-65504.0)
    W[11, 8] = np.float16(6.1e-5)
    rng = np.random.default_rng(5)
    W[12:] = rng.standard_normal((M - 12, K)).astype(np.float16) * np.float16(0.02)
    return W


@pytest.mark.parametrize("M,K,seed", [(256, 512, 0), (16, 256, 1), (80, 1280, 2), (48, 2304, 3)])
def test_quantize_pack_bit_exact(pkg, o5, wd, M, K, seed):
    _say(wd.prefix + " quantize_pack M=%d K=%d seed=%d" % (M, K, seed))
    W = workloads.make_weights(M, K, seed)
    packed, scales = _call(pkg, wd, "quantize_pack")(W.cuda())
    torch.cuda.synchronize()
    ref_packed, ref_scales = o5.quantize_pack(W.numpy())
    assert packed.numel() == o5.packed_bytes(M, K) == wd.bits * 16 * wd.tile_cols // 8 * (M // 16) * -(-K // wd.tile_cols)
    assert np.array_equal(_np(scales).view(np.uint16), ref_scales.view(np.uint16))
    assert np.array_equal(_np(packed), ref_packed)


def test_quantize_pack_special_values(pkg, o5, wd):
    _say(wd.prefix + " quantize_pack special values")
    W = _special_matrix(o5, wd)
    M, K = W.shape
    packed, scales = _call(pkg, wd, "quantize_pack")(torch.from_numpy(W).cuda())
    torch.cuda.synchronize()
    ref_packed, ref_scales = o5.quantize_pack(W)
    assert np.array_equal(_np(scales).view(np.uint16), ref_scales.view(np.uint16))
    got_codes = o5.unpack_codes(_np(packed), M, K)
    assert np.array_equal(got_codes, o5.unpack_codes(ref_packed, M, K))
    assert np.array_equal(_np(packed), ref_packed)
    assert np.array_equal(got_codes[0, :wd.codes], np.arange(wd.codes, dtype=np.uint8))
    back = _call(pkg, wd, "unpack")(packed, scales, M, K)
    torch.cuda.synchronize()
    assert np.array_equal(_np(back).view(np.uint16), o5.unpack(ref_packed, ref_scales, M, K).view(np.uint16))


def test_unpack_every_code_and_scales(pkg, o5, wd):
    """All codes at every position of a lane's group under assorted scales: bit-exact, signed zeros kept."""
    _say(wd.prefix + " unpack every code")
    M, K = 16, 256
    codes = np.zeros((M, K), dtype=np.uint8)
    for m in range(M):
        codes[m] = (np.arange(K) * (2 * m + 1) + m) % wd.codes
    scale_bits = np.array([0x3C00, 0x0000, 0x0001, 0x0002, 0x03FF, 0x0400, 0x1E00, 0x2001, 0x77FF, 0x68AB,
                           0x0155, 0x2E66, 0x3555, 0x1001, 0x5BFF, 0x7BFF], dtype=np.uint16)
    packed = o5.pack(codes)
    scales = scale_bits.view(np.float16)
    got = _call(pkg, wd, "unpack")(torch.from_numpy(packed).cuda(), torch.from_numpy(scales.copy()).cuda(), M, K)
    torch.cuda.synchronize()
    want = o5.unpack(packed, scales, M, K)
    assert np.array_equal(_np(got).view(np.uint16), want.view(np.uint16))
    assert np.isinf(want.astype(np.float32)).any()      # top * 65504 overflows: inf on both sides


def _linear_case(pkg, o5, wd, M, K, N, seed, split=0):
    W = workloads.make_weights(M, K, seed).numpy()
    X = workloads.make_activations(N, K, seed)
    packed, scales = o5.quantize_pack(W)
    pkg.fp6_tuning_set_split_k(split)
    try:
        Y = _call(pkg, wd, "linear")(torch.from_numpy(packed).cuda(), torch.from_numpy(scales).cuda(), X.cuda(), M, K)
        torch.cuda.synchronize()
    finally:
        pkg.fp6_tuning_set_split_k(0)
    return _np(Y), o5.linear(packed, scales, X.numpy(), M, K)


@pytest.mark.parametrize("N", [1, 3, 8, 16, 17, 32, 33, 64, 70, 130, 257])
def test_linear_token_counts(pkg, o5, wd, N):
    M, K = 80, 1280
    _say(wd.prefix + " linear M=%d K=%d N=%d" % (M, K, N))
    Y, Y_ref = _linear_case(pkg, o5, wd, M, K, N, seed=N)
    worst = _check_linear(Y, Y_ref, "N=%d" % N)
    assert worst < 2e-3


@pytest.mark.parametrize("split", [1, 2, 3, 5])
@pytest.mark.parametrize("N", [5, 48, 100])
def test_linear_split_k(pkg, o5, wd, split, N):
    M, K = 144, 2816
    _say(wd.prefix + " linear split-K S=%d N=%d" % (split, N))
    Y, Y_ref = _linear_case(pkg, o5, wd, M, K, N, seed=split, split=split)
    _check_linear(Y, Y_ref, "split=%d" % split)


def test_linear_exact_cases_and_determinism(pkg, o5, wd):
    _say(wd.prefix + " linear exact cases")
    M, K, N = 64, 1024, 9
    X = workloads.make_activations(N, K, seed=1)
    # one non-zero v = top * 2^-k (or top * 0.1875) per row: the result is v * X[pi(m)], exact after one fp16 rounding
    W = np.zeros((M, K), dtype=np.float16)
    pi = (np.arange(M) * 37 + 5) % K
    W[np.arange(M), pi] = wd.unit
    packed, scales = _call(pkg, wd, "quantize_pack")(torch.from_numpy(W).cuda())
    Y = _call(pkg, wd, "linear")(packed, scales, X.cuda(), M, K)
    torch.cuda.synchronize()
    want = (wd.unit * X.numpy().astype(np.float64)[:, pi]).astype(np.float16)
    assert np.array_equal(_np(Y).view(np.uint16), want.view(np.uint16))
    # reruns give identical bits
    Wr = workloads.make_weights(M, K, 3).cuda()
    packed, scales = _call(pkg, wd, "quantize_pack")(Wr)
    outs = [_call(pkg, wd, "linear")(packed, scales, X.cuda(), M, K) for _ in range(4)]
    torch.cuda.synchronize()
    for o in outs[1:]:
        assert torch.equal(o.view(torch.int16), outs[0].view(torch.int16))


def test_full_size_layer_sampled(pkg, o5, wd):
    """The benchmark layer at its real size: packed stream and scales bit for bit on sampled row tiles, Y on their rows."""
    name, M, K = workloads.FFN_65B
    _say(wd.prefix + " full-size %s M=%d K=%d" % (name, M, K))
    W = workloads.make_weights(M, K, seed=0, device="cuda")
    packed, scales = _call(pkg, wd, "quantize_pack")(W)
    torch.cuda.synchronize()
    rng = np.random.default_rng(1)
    tiles = np.array(sorted(set([0, M // 16 - 1]) | set(int(t) for t in rng.choice(M // 16, size=14, replace=False))))
    rows = (tiles[:, None] * 16 + np.arange(16)[None, :]).ravel()
    ref_packed, ref_scales = o5.quantize_pack(_np(W[torch.from_numpy(rows).cuda()]))
    got_packed = row_tiles_of(packed, M, K, tiles, wd.tile_bytes, wd.tile_cols)
    assert np.array_equal(_np(scales)[rows].view(np.uint16), ref_scales.view(np.uint16))
    assert np.array_equal(got_packed, ref_packed)
    del W
    for N in (1, 16, 32, 512):
        _say("  " + wd.prefix + " linear N=%d" % N)
        X = workloads.make_activations(N, K, seed=N, device="cuda")
        Y = _call(pkg, wd, "linear")(packed, scales, X, M, K)
        torch.cuda.synchronize()
        Y_ref = o5.linear(ref_packed, ref_scales, _np(X), len(rows), K)
        _check_linear(_np(Y)[:, rows], Y_ref, "%s N=%d" % (name, N))
