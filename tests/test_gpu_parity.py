"""GPU parity tests: the HIP path, called through the C-ABI binding, against the CPU oracle.

pack / unpack are compared bit for bit; the GEMM must satisfy, for every output column n,
max_m |Y_gpu - Y_ref| <= 5e-3 * max_m |Y_ref| (Y_ref in fp64).
"""
import numpy as np
import pytest
import torch

import workloads
from gpu_checks import check_linear as _check_linear
from packed_rows import row_tiles_of

pytestmark = pytest.mark.gpu



@pytest.fixture(scope="module")
def pkg():
    import paper_2401_14112_amd as p

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    p.load_library()
    return p


def _say(msg):
    print(msg, flush=True)


def _np16(t):
    return t.detach().cpu().numpy()


# ------------------------------------------------------------------ pack / unpack
@pytest.mark.parametrize("M,K,seed", [(256, 512, 0), (16, 256, 1), (80, 1280, 2), (48, 2304, 3)])
def test_quantize_pack_bit_exact(pkg, oracle, M, K, seed):
    _say("quantize_pack M=%d K=%d seed=%d" % (M, K, seed))
    W = workloads.make_weights(M, K, seed)
    packed, scales = pkg.fp6_quantize_pack(W.cuda())
    torch.cuda.synchronize()
    ref_packed, ref_scales = oracle.quantize_pack(W.numpy())
    assert np.array_equal(_np16(scales).view(np.uint16), ref_scales.view(np.uint16))
    assert np.array_equal(_np16(packed), ref_packed)


def _special_matrix(oracle):
    """Rows that exercise every code, ties, signed zeros, zero rows and rows with subnormal scales."""
    table = oracle.decode_table()
    M, K = 32, 512
    W = np.zeros((M, K), dtype=np.float16)
    for m, s in enumerate([2.0 ** -6, 0.01171875, 1.0, 3.0]):
        W[m, :64] = (table * s).astype(np.float16)
        W[m, 100:164] = (table[::-1] * s).astype(np.float16)
    ties = [26, 22, 18, 1.875, 0.21875, 0.09375, 0.03125, 27, 25, 1.1, 1.13, 0.04, 0.03]
    W[4, 0] = 28.0
    W[4, 1:1 + len(ties)] = ties
    W[5, 0] = -28.0
    W[5, 1:1 + len(ties)] = [-t for t in ties]
    W[6, 3] = -0.0                                   # all-zero row with one negative zero
    W[7, :] = np.float16(2.0 ** -24)                 # scale rounds to zero
    W[7, 5] = -np.float16(2.0 ** -24)
    W[8, 0] = np.float16(28 * 2.0 ** -24)            # subnormal scale 2^-24
    W[8, 1] = np.float16(14 * 2.0 ** -24)
    W[8, 2] = -np.float16(3 * 2.0 ** -24)
    W[9, 0] = np.float16(41 * 2.0 ** -24)            # scale rounds down so the row maximum saturates
    W[9, 1] = np.float16(13 * 2.0 ** -24)
    W[10, :] = np.float16(65504.0)                   # largest fp16 everywhere
    W[11, 7] = np.float16(-65504.0)
    W[11, 8] = np.float16(6.1e-5)
    rng = np.random.default_rng(5)
    W[12:] = rng.standard_normal((M - 12, K)).astype(np.float16) * np.float16(0.02)
    return W


def test_quantize_pack_special_values(pkg, oracle):
    _say("quantize_pack special values")
    W = _special_matrix(oracle)
    M, K = W.shape
    packed, scales = pkg.fp6_quantize_pack(torch.from_numpy(W).cuda())
    torch.cuda.synchronize()
    ref_packed, ref_scales = oracle.quantize_pack(W)
    assert np.array_equal(_np16(scales).view(np.uint16), ref_scales.view(np.uint16))
    got_codes = oracle.unpack_codes(_np16(packed), M, K)
    ref_codes = oracle.unpack_codes(ref_packed, M, K)
    assert np.array_equal(got_codes, ref_codes)
    assert np.array_equal(_np16(packed), ref_packed)
    # the every-code rows come back as the codes 0..63
    assert np.array_equal(got_codes[0, :64], np.arange(64, dtype=np.uint8))


@pytest.mark.parametrize("M,K,seed", [(256, 512, 0), (80, 1280, 2)])
def test_unpack_bit_exact(pkg, oracle, M, K, seed):
    _say("unpack M=%d K=%d" % (M, K))
    W = workloads.make_weights(M, K, seed).numpy()
    ref_packed, ref_scales = oracle.quantize_pack(W)
    got = pkg.fp6_unpack(torch.from_numpy(ref_packed).cuda(), torch.from_numpy(ref_scales).cuda(), M, K)
    torch.cuda.synchronize()
    want = oracle.unpack(ref_packed, ref_scales, M, K)
    assert np.array_equal(_np16(got).view(np.uint16), want.view(np.uint16))


def test_unpack_every_code_and_scales(pkg, oracle):
    """All 64 codes under assorted scales (normal, subnormal, zero, large): bit-exact, signed zeros kept."""
    _say("unpack every code")
    M, K = 16, 256
    codes = np.zeros((M, K), dtype=np.uint8)
    for m in range(M):
        codes[m] = (np.arange(K) * (2 * m + 1) + m) % 64
    scale_bits = np.array([0x3C00, 0x0000, 0x0001, 0x0002, 0x03FF, 0x0400, 0x1E00, 0x2001, 0x77FF, 0x68AB,
                           0x0155, 0x2E66, 0x3555, 0x1001, 0x5BFF, 0x63FF], dtype=np.uint16)
    packed = oracle.pack(codes)
    scales = scale_bits.view(np.float16)
    got = pkg.fp6_unpack(torch.from_numpy(packed).cuda(), torch.from_numpy(scales.copy()).cuda(), M, K)
    torch.cuda.synchronize()
    want = oracle.unpack(packed, scales, M, K)
    assert np.array_equal(_np16(got).view(np.uint16), want.view(np.uint16))
    assert np.isinf(want.astype(np.float32)).any()      # 28 * 32752 overflows: rounded to inf on both sides


def test_pack_then_unpack_on_gpu(pkg, oracle):
    _say("pack -> unpack round trip on the GPU")
    W = _special_matrix(oracle)
    M, K = W.shape
    packed, scales = pkg.fp6_quantize_pack(torch.from_numpy(W).cuda())
    back = pkg.fp6_unpack(packed, scales, M, K)
    torch.cuda.synchronize()
    ref_packed, ref_scales = oracle.quantize_pack(W)
    want = oracle.unpack(ref_packed, ref_scales, M, K)
    assert np.array_equal(_np16(back).view(np.uint16), want.view(np.uint16))


# ------------------------------------------------------------------ linear
def _linear_case(pkg, oracle, M, K, N, seed, split=0, x_scale=1.0):
    W = workloads.make_weights(M, K, seed).numpy()
    X = (workloads.make_activations(N, K, seed) * x_scale).to(torch.float16)
    packed, scales = oracle.quantize_pack(W)
    pkg.fp6_tuning_set_split_k(split)
    try:
        Y = pkg.fp6_linear(torch.from_numpy(packed).cuda(), torch.from_numpy(scales).cuda(), X.cuda(), M, K)
        torch.cuda.synchronize()
    finally:
        pkg.fp6_tuning_set_split_k(0)
    Y_ref = oracle.linear(packed, scales, X.numpy(), M, K)
    return _np16(Y), Y_ref


def test_linear_config1(pkg, oracle):
    name, M, K = workloads.TINY
    _say("linear tiny config M=%d K=%d N=8" % (M, K))
    Y, Y_ref = _linear_case(pkg, oracle, M, K, 8, seed=0)
    worst = _check_linear(Y, Y_ref, "tiny")
    _say("  worst column ratio %.3g" % worst)
    assert worst < 2e-3          # fp32 accumulation: the error is the final fp16 rounding


@pytest.mark.parametrize("N", [1, 2, 3, 4, 7, 8, 15, 16, 17, 24, 31, 32, 33, 48, 70])
def test_linear_token_counts(pkg, oracle, N):
    M, K = 80, 1280          # 5 row tiles (ragged against 4 waves per block), 5 k-tiles
    _say("linear M=%d K=%d N=%d" % (M, K, N))
    Y, Y_ref = _linear_case(pkg, oracle, M, K, N, seed=N)
    _check_linear(Y, Y_ref, "N=%d" % N)


@pytest.mark.parametrize("M,K,N", [(10256, 1536, 5), (10240, 1536, 16), (28672, 512, 3)])
def test_linear_tall_stream_blocks(pkg, oracle, M, K, N):
    """Shapes for which the plan takes the 8-wave block of the N <= 16 streaming kernel (more blocks fit one
    round than with 4-wave blocks), with and without a ragged last block and with / without split-K."""
    _say("tall stream blocks M=%d K=%d N=%d" % (M, K, N))
    W = workloads.make_weights(M, K, seed=11)
    packed, scales = oracle.quantize_pack(_np16(W))
    X = workloads.make_activations(N, K, seed=N)
    Y = pkg.fp6_linear(torch.from_numpy(packed).cuda(), torch.from_numpy(scales).cuda(), X.cuda(), M, K)
    torch.cuda.synchronize()
    _check_linear(_np16(Y), oracle.linear(packed, scales, _np16(X), M, K), "tall blocks")


@pytest.mark.parametrize("split", [1, 2, 3, 5, 64])
@pytest.mark.parametrize("N", [5, 32])
def test_linear_split_k(pkg, oracle, split, N):
    M, K = 144, 2816         # 9 row tiles, 11 k-tiles
    _say("linear split-K S=%d N=%d" % (split, N))
    Y, Y_ref = _linear_case(pkg, oracle, M, K, N, seed=split, split=split)
    _check_linear(Y, Y_ref, "split=%d" % split)


def test_linear_is_deterministic_and_workspace_reusable(pkg, oracle):
    M, K, N = 256, 4096, 16
    _say("linear determinism / workspace reuse")
    W = workloads.make_weights(M, K, 3).cuda()
    X = workloads.make_activations(N, K, 3).cuda()
    packed, scales = pkg.fp6_quantize_pack(W)
    pkg.fp6_tuning_set_split_k(4)
    try:
        nbytes = pkg.fp6_linear_workspace_bytes(M, N, K)
        assert nbytes > 0
        ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")
        pkg.fp6_workspace_init(ws)
        outs = []
        for _ in range(5):
            outs.append(pkg.fp6_linear(packed, scales, X, M, K, workspace=ws).clone())
        torch.cuda.synchronize()
    finally:
        pkg.fp6_tuning_set_split_k(0)
    for o in outs[1:]:
        assert torch.equal(o.view(torch.int16), outs[0].view(torch.int16))
    Y_ref = oracle.linear(_np16(packed), _np16(scales), _np16(X), M, K)
    _check_linear(_np16(outs[0]), Y_ref, "reuse")


def test_linear_exact_special_cases(pkg, oracle):
    """Cases with a closed form that the GPU must hit exactly after its single fp16 rounding."""
    _say("linear closed-form cases")
    M, K, N = 48, 512, 4
    rng = np.random.default_rng(11)
    pi = rng.permutation(K)[:M]
    sign = rng.choice([-1.0, 1.0], M)
    W = np.zeros((M, K), dtype=np.float16)
    W[np.arange(M), pi] = (0.875 * sign).astype(np.float16)
    X = workloads.make_activations(N, K, 4)
    packed, scales = pkg.fp6_quantize_pack(torch.from_numpy(W).cuda())
    Y = pkg.fp6_linear(packed, scales, X.cuda(), M, K)
    torch.cuda.synchronize()
    want = (0.875 * sign[None, :] * X.numpy().astype(np.float64)[:, pi]).astype(np.float16)
    assert np.array_equal(_np16(Y).view(np.uint16), want.view(np.uint16))
    # subnormal codes only (E = 0): a flush of fp16 subnormals anywhere in the unpack would zero these
    codes = np.full((M, K), 0b000011, dtype=np.uint8)          # 3/16
    codes[:, ::2] = 0b100001                                    # -1/16
    scales1 = np.ones(M, dtype=np.float16)
    Xs = torch.ones((N, K), dtype=torch.float16)
    Y2 = pkg.fp6_linear(torch.from_numpy(oracle.pack(codes)).cuda(), torch.from_numpy(scales1).cuda(), Xs.cuda(), M, K)
    torch.cuda.synchronize()
    assert np.all(_np16(Y2).astype(np.float64) == (K // 2) * (3 / 16 - 1 / 16))


def test_linear_all_codes_against_oracle(pkg, oracle):
    _say("linear with uniformly random codes and assorted scales")
    M, K, N = 64, 1024, 9
    codes = workloads.make_codes(M, K, 21).numpy()
    scales = (np.abs(np.random.default_rng(2).standard_normal(M)) * 0.01 + 1e-4).astype(np.float16)
    X = workloads.make_activations(N, K, 21)
    packed = oracle.pack(codes)
    Y = pkg.fp6_linear(torch.from_numpy(packed).cuda(), torch.from_numpy(scales).cuda(), X.cuda(), M, K)
    torch.cuda.synchronize()
    _check_linear(_np16(Y), oracle.linear_codes(codes, scales, X.numpy()), "all codes")


@pytest.mark.parametrize("N", [1, 8, 32, 40])
def test_fp16_linear(pkg, oracle, N):
    M, K = 80, 1280
    _say("fp16_linear M=%d K=%d N=%d" % (M, K, N))
    W = workloads.make_weights(M, K, 7)
    X = workloads.make_activations(N, K, 7)
    Y = pkg.fp16_linear(W.cuda(), X.cuda())
    torch.cuda.synchronize()
    _check_linear(_np16(Y), oracle.linear_f16(W.numpy(), X.numpy()), "fp16 N=%d" % N)


@pytest.mark.parametrize("N", [3, 16, 32, 64])
@pytest.mark.parametrize("split", [2, 3, 5])
def test_fp16_linear_stream_forced_split(pkg, oracle, N, split):
    """The fp16 weight tiles of the streaming kernel pass through LDS: every shape of that kernel (1, 2, 4 token
    tiles per wave; 4- and 8-wave blocks with a ragged last block) under split-K factors that do not divide
    the 11 k-tiles, twice for identical bits."""
    M, K = 272, 2816
    _say("fp16_linear stream M=%d K=%d N=%d split=%d" % (M, K, N, split))
    W = workloads.make_weights(M, K, 11)
    X = workloads.make_activations(N, K, 11)
    pkg.fp6_tuning_set_split_k(split)
    try:
        Y = pkg.fp16_linear(W.cuda(), X.cuda())
        Y2 = pkg.fp16_linear(W.cuda(), X.cuda())
        torch.cuda.synchronize()
    finally:
        pkg.fp6_tuning_set_split_k(0)
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16))
    _check_linear(_np16(Y), oracle.linear_f16(W.numpy(), X.numpy()), "fp16 stream N=%d split=%d" % (N, split))


# ------------------------------------------------------------------ tiled kernel (N > 32)
@pytest.mark.parametrize("rt,nt", [(0, 0), (128, 64), (256, 64), (128, 128), (256, 128)])
@pytest.mark.parametrize("N,split", [(33, 1), (64, 0), (100, 2), (128, 3), (257, 0)])
def test_linear_tiled(pkg, oracle, rt, nt, N, split):
    M, K = 272, 2816         # 17 row tiles (ragged against every block height), 11 k-tiles
    _say("tiled linear block=%dx%d N=%d split=%d" % (rt, nt, N, split))
    pkg.fp6_tuning_set_tile(rt, nt)
    try:
        Y, Y_ref = _linear_case(pkg, oracle, M, K, N, seed=N + rt, split=split)
    finally:
        pkg.fp6_tuning_set_tile(0, 0)
    _check_linear(Y, Y_ref, "tiled rt=%d nt=%d N=%d" % (rt, nt, N))


@pytest.mark.parametrize("rt,nt", [(0, 0), (128, 64), (128, 128), (256, 128)])
@pytest.mark.parametrize("N,split", [(64, 0), (130, 2)])
def test_fp16_linear_tiled(pkg, oracle, rt, nt, N, split):
    M, K = 272, 2816
    _say("tiled fp16_linear rt=%d nt=%d N=%d split=%d" % (rt, nt, N, split))
    W = workloads.make_weights(M, K, 7)
    X = workloads.make_activations(N, K, 7)
    pkg.fp6_tuning_set_tile(rt, nt)
    pkg.fp6_tuning_set_split_k(split)
    try:
        Y = pkg.fp16_linear(W.cuda(), X.cuda())
        torch.cuda.synchronize()
    finally:
        pkg.fp6_tuning_set_tile(0, 0)
        pkg.fp6_tuning_set_split_k(0)
    _check_linear(_np16(Y), oracle.linear_f16(W.numpy(), X.numpy()), "tiled fp16 N=%d" % N)


def test_tiled_deterministic_and_exact_cases(pkg, oracle):
    _say("tiled: determinism and subnormal codes")
    M, K, N = 256, 4096, 96
    W = workloads.make_weights(M, K, 3).cuda()
    X = workloads.make_activations(N, K, 3).cuda()
    packed, scales = pkg.fp6_quantize_pack(W)
    pkg.fp6_tuning_set_split_k(4)
    try:
        nbytes = pkg.fp6_linear_workspace_bytes(M, N, K)
        assert nbytes > 0
        ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
        outs = [pkg.fp6_linear(packed, scales, X, M, K, workspace=ws).clone() for _ in range(4)]
        torch.cuda.synchronize()
    finally:
        pkg.fp6_tuning_set_split_k(0)
    for o in outs[1:]:
        assert torch.equal(o.view(torch.int16), outs[0].view(torch.int16))
    _check_linear(_np16(outs[0]), oracle.linear(_np16(packed), _np16(scales), _np16(X), M, K), "tiled reuse")
    codes = np.full((M, K), 0b000011, dtype=np.uint8)
    codes[:, ::2] = 0b100001
    Y2 = pkg.fp6_linear(torch.from_numpy(oracle.pack(codes)).cuda(), torch.ones(M, dtype=torch.float16).cuda(),
                        torch.ones((N, K), dtype=torch.float16).cuda(), M, K)
    torch.cuda.synchronize()
    assert np.all(_np16(Y2).astype(np.float64) == (K // 2) * (3 / 16 - 1 / 16))


# ------------------------------------------------------------------ full-size layer, sampled rows
def _sampled_row_tiles(M, count, seed):
    rng = np.random.default_rng(seed)
    tiles = set([0, M // 16 - 1])
    tiles.update(int(t) for t in rng.choice(M // 16, size=count - 2, replace=False))
    return np.array(sorted(tiles), dtype=np.int64)


@pytest.mark.parametrize("shape", [workloads.FFN_65B, workloads.FFN_65B_DOWN])
def test_full_size_layer_sampled(pkg, oracle, shape):
    """The benchmark layer at its real size, in the launch configuration bench.py times: the packed
    stream and scales are compared bit for bit on sampled 16-row tiles (the tiles of a row tile are gathered from the
    stream), and Y on the rows of those tiles for N = 1 ... 512 (every kernel
    and block shape the plan picks for this layer)."""
    name, M, K = shape
    _say("full-size %s M=%d K=%d" % (name, M, K))
    W = workloads.make_weights(M, K, seed=0, device="cuda")
    packed, scales = pkg.fp6_quantize_pack(W)
    torch.cuda.synchronize()
    tiles = _sampled_row_tiles(M, 24, seed=1)
    rows = (tiles[:, None] * 16 + np.arange(16)[None, :]).ravel()
    W_rows = _np16(W[torch.from_numpy(rows).cuda()])
    ref_packed, ref_scales = oracle.quantize_pack(W_rows)          # the sampled tiles as a 16*T-row matrix
    got_packed = row_tiles_of(packed, M, K, tiles, 3072)
    assert np.array_equal(_np16(scales)[rows].view(np.uint16), ref_scales.view(np.uint16))
    assert np.array_equal(got_packed, ref_packed)
    del W
    for N in (1, 8, 16, 32, 64, 128, 256, 512):
        _say("  linear N=%d" % N)
        X = workloads.make_activations(N, K, seed=N, device="cuda")
        Y = pkg.fp6_linear(packed, scales, X, M, K)
        torch.cuda.synchronize()
        Y_ref = oracle.linear(ref_packed, ref_scales, _np16(X), len(rows), K)
        worst = _check_linear(_np16(Y)[:, rows], Y_ref, "%s N=%d" % (name, N))
        _say("    worst column ratio %.3g" % worst)
        # every output was written: no row of Y may still hold the fill pattern of a fresh buffer
        Yf = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
        pkg.fp6_linear(packed, scales, X, M, K, out=Yf)
        torch.cuda.synchronize()
        assert not torch.isnan(Yf).any()
        assert torch.equal(Yf.view(torch.int16), Y.view(torch.int16))


@pytest.mark.parametrize("shape", [workloads.FFN_65B, workloads.FFN_65B_DOWN])
def test_fp16_linear_full_size_sampled(pkg, oracle, shape):
    """The library's own fp16-weight layer at the shapes it is timed on (both orientations of the benchmark
    layer), on sampled row tiles, for the token counts of every kernel it dispatches to."""
    name, M, K = shape
    _say("fp16_linear full-size %s M=%d K=%d" % (name, M, K))
    W = workloads.make_weights(M, K, seed=0, device="cuda")
    tiles = _sampled_row_tiles(M, 16, seed=2)
    rows = (tiles[:, None] * 16 + np.arange(16)[None, :]).ravel()
    W_rows = _np16(W[torch.from_numpy(rows).cuda()])
    for N in (1, 16, 32, 64, 128, 512):
        _say("  fp16_linear N=%d" % N)
        X = workloads.make_activations(N, K, seed=N, device="cuda")
        Y = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
        pkg.fp16_linear(W, X, out=Y)
        torch.cuda.synchronize()
        assert not torch.isnan(Y).any()
        worst = _check_linear(_np16(Y)[:, rows], oracle.linear_f16(W_rows, _np16(X)), "fp16 %s N=%d" % (name, N))
        _say("    worst column ratio %.3g" % worst)


def test_largest_admitted_matrix_offsets(pkg, oracle):
    """Tiles are stored k-tile major and addressed with 32-bit offsets that span the whole matrix: a tall
    matrix just inside the limit (K/256 + 64) * (M/16) * 3072 < 2^31 puts a wave's last tiles 680 MB past its
    first and its out-of-range look-ahead close to 2^31.  Packed stream and scales bit for bit on sampled row
    tiles (first, last, random), Y on their rows, for the streaming kernel and the tiled one, and the round
    trip through fp6_unpack on those rows; the next size up is refused."""
    M, K = 114688, 8192
    assert (K // 256 + 64) * (M // 16) * 3072 < 2 ** 31 <= (K // 256 + 64) * ((M + 2048) // 16) * 3072
    _say("largest admitted matrix M=%d K=%d" % (M, K))
    W = workloads.make_weights(M, K, seed=11, device="cuda")
    packed, scales = pkg.fp6_quantize_pack(W)
    torch.cuda.synchronize()
    tiles = _sampled_row_tiles(M, 12, seed=5)
    rows = (tiles[:, None] * 16 + np.arange(16)[None, :]).ravel()
    ref_packed, ref_scales = oracle.quantize_pack(_np16(W[torch.from_numpy(rows).cuda()]))
    del W
    assert np.array_equal(row_tiles_of(packed, M, K, tiles, 3072), ref_packed)
    assert np.array_equal(_np16(scales)[rows].view(np.uint16), ref_scales.view(np.uint16))
    Wd = pkg.fp6_unpack(packed, scales, M, K)
    torch.cuda.synchronize()
    want = oracle.unpack(ref_packed, ref_scales, len(rows), K)
    assert np.array_equal(_np16(Wd[torch.from_numpy(rows).cuda()]).view(np.uint16), want.view(np.uint16))
    del Wd
    for N in (1, 32, 128):
        _say("  linear N=%d" % N)
        X = workloads.make_activations(N, K, seed=N, device="cuda")
        Y = pkg.fp6_linear(packed, scales, X, M, K)
        torch.cuda.synchronize()
        Y_ref = oracle.linear(ref_packed, ref_scales, _np16(X), len(rows), K)
        _check_linear(_np16(Y)[:, rows], Y_ref, "largest matrix N=%d" % N)
        assert not torch.isnan(Y).any()
    with pytest.raises(pkg.Fp6Error):
        pkg.fp6_linear(packed, scales, X, M + 2048, K)


# ------------------------------------------------------------------ 70B-class layer set, decoder weight stream
def _sampled_reference(pkg, oracle, W, packed, scales, M, K, count, seed):
    """Oracle-side packed stream and scales of `count` sampled 16-row tiles, after checking that the
    library's packed stream and scales on those tiles are the same bytes."""
    tiles = _sampled_row_tiles(M, count, seed)
    rows = (tiles[:, None] * 16 + np.arange(16)[None, :]).ravel()
    ref_packed, ref_scales = oracle.quantize_pack(_np16(W[torch.from_numpy(rows).cuda()]))
    got_packed = row_tiles_of(packed, M, K, tiles, 3072)
    assert np.array_equal(_np16(scales)[rows].view(np.uint16), ref_scales.view(np.uint16))
    assert np.array_equal(got_packed, ref_packed)
    return rows, ref_packed, ref_scales


@pytest.mark.parametrize("shape", workloads.SET_70B)
def test_layer_set_70b(pkg, oracle, shape):
    """The four linear layers of a 70B-class decoder block at N = 16, real sizes, sampled row tiles."""
    name, M, K = shape
    _say("layer set %s M=%d K=%d N=16" % (name, M, K))
    W = workloads.make_weights(M, K, seed=7, device="cuda")
    packed, scales = pkg.fp6_quantize_pack(W)
    torch.cuda.synchronize()
    rows, ref_packed, ref_scales = _sampled_reference(pkg, oracle, W, packed, scales, M, K, 16, seed=2)
    del W
    X = workloads.make_activations(16, K, seed=16, device="cuda")
    Y = pkg.fp6_linear(packed, scales, X, M, K)
    torch.cuda.synchronize()
    worst = _check_linear(_np16(Y)[:, rows], oracle.linear(ref_packed, ref_scales, _np16(X), len(rows), K), name)
    _say("  worst column ratio %.3g" % worst)


@pytest.mark.parametrize("N", [1, 32])
def test_decoder_weight_stream_graph(pkg, oracle, N):
    """80 GEMMs (20 decoder blocks x the four layer shapes, every GEMM with packed weights of its own) captured
    into one HIP graph and replayed three times with eager work in between; every replay must give the bits
    of the eager launches, and sampled rows of one GEMM per shape must agree with the oracle."""
    blocks = 20
    layers = []      # (name, M, K, packed, scales, X, Y, ws)
    refs = {}
    for b in range(blocks):
        for j, (name, M, K) in enumerate(workloads.SET_70B):
            W = workloads.make_weights(M, K, seed=1000 + 4 * b + j, device="cuda")
            packed, scales = pkg.fp6_quantize_pack(W)
            if b == blocks - 1:
                torch.cuda.synchronize()
                refs[len(layers)] = _sampled_reference(pkg, oracle, W, packed, scales, M, K, 6, seed=3 + j)
            del W
            X = workloads.make_activations(N, K, seed=50 + j, device="cuda")
            Y = torch.empty((N, M), dtype=torch.float16, device="cuda")
            ws = torch.zeros(max(pkg.fp6_linear_workspace_bytes(M, N, K), 16), dtype=torch.uint8, device="cuda")
            layers.append((name, M, K, packed, scales, X, Y, ws))
    _say("decoder stream N=%d: %d GEMMs, %.2f GB packed" % (N, len(layers), sum(l[3].numel() for l in layers) * 1e-9))

    def run_all():
        for name, M, K, packed, scales, X, Y, ws in layers:
            pkg.fp6_linear(packed, scales, X, M, K, out=Y, workspace=ws)

    run_all()
    torch.cuda.synchronize()
    eager = [l[6].clone() for l in layers]
    for i, (rows, ref_packed, ref_scales) in refs.items():
        name, M, K, _, _, X, Y, _ = layers[i]
        _check_linear(_np16(Y)[:, rows], oracle.linear(ref_packed, ref_scales, _np16(X), len(rows), K), name)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run_all()
    for replay in range(3):
        for l in layers:
            l[6].fill_(float("nan"))          # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for l, e in zip(layers, eager):
            assert torch.equal(l[6].view(torch.int16), e.view(torch.int16)), "replay %d, %s" % (replay, l[0])


def test_linear_more_tokens_than_one_launch_can_address(pkg, oracle):
    """Activations larger than 2 GiB (the kernels address them with 32-bit byte offsets): the call is cut into
    launches of at most floor((2^31 - 1) / 2K) tokens rounded down to 128.  Sampled tokens around the cut,
    at both ends and in the short last piece against the oracle; every output written."""
    M, K = 32, 256
    chunk = ((2 ** 31 - 1) // (2 * K)) // 128 * 128
    N = chunk + 300
    _say("linear M=%d K=%d N=%d (two launches: %d + 300 tokens)" % (M, K, N, chunk))
    W = workloads.make_weights(M, K, seed=9)
    packed, scales = oracle.quantize_pack(W.numpy())
    X = workloads.make_activations(N, K, seed=77, device="cuda")
    assert X.numel() * 2 > 2 ** 31
    Y = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    pkg.fp6_linear(torch.from_numpy(packed).cuda(), torch.from_numpy(scales).cuda(), X, M, K, out=Y)
    torch.cuda.synchronize()
    assert not torch.isnan(Y).any()
    rng = np.random.default_rng(4)
    tokens = np.unique(np.concatenate([np.arange(0, 40), np.arange(chunk - 130, chunk + 130), np.arange(N - 40, N),
                                       rng.integers(0, N, size=64)]))
    idx = torch.from_numpy(tokens).cuda()
    Y_ref = oracle.linear(packed, scales, _np16(X[idx]), M, K)
    _check_linear(_np16(Y[idx]), Y_ref, "long input")


def test_linear_two_streams_with_their_own_workspaces(pkg, oracle):
    """Calls that overlap on the GPU (two streams) with a workspace each give the bits of the same calls made
    one after the other; split-K is forced so that both use partial tiles and arrival counters."""
    M, K = 512, 4096
    _say("linear on two streams M=%d K=%d" % (M, K))
    Wa = workloads.make_weights(M, K, 31).cuda()
    Wb = workloads.make_weights(M, K, 32).cuda()
    pa, sa = pkg.fp6_quantize_pack(Wa)
    pb, sb = pkg.fp6_quantize_pack(Wb)
    pkg.fp6_tuning_set_split_k(4)
    try:
        cases = []
        for N in (4, 48, 200):
            Xa = workloads.make_activations(N, K, N).cuda()
            Xb = workloads.make_activations(N, K, N + 1).cuda()
            nbytes = max(pkg.fp6_linear_workspace_bytes(M, N, K), 16)
            wsa = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
            wsb = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
            ref_a = pkg.fp6_linear(pa, sa, Xa, M, K, workspace=wsa).clone()
            ref_b = pkg.fp6_linear(pb, sb, Xb, M, K, workspace=wsb).clone()
            torch.cuda.synchronize()
            s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
            outs_a, outs_b = [], []
            for _ in range(6):
                with torch.cuda.stream(s1):
                    outs_a.append(pkg.fp6_linear(pa, sa, Xa, M, K, workspace=wsa).clone())
                with torch.cuda.stream(s2):
                    outs_b.append(pkg.fp6_linear(pb, sb, Xb, M, K, workspace=wsb).clone())
            torch.cuda.synchronize()
            for o in outs_a:
                assert torch.equal(o.view(torch.int16), ref_a.view(torch.int16))
            for o in outs_b:
                assert torch.equal(o.view(torch.int16), ref_b.view(torch.int16))
            cases.append((N, Xa, ref_a))
    finally:
        pkg.fp6_tuning_set_split_k(0)
    N, Xa, ref_a = cases[1]
    _check_linear(_np16(ref_a), oracle.linear(_np16(pa), _np16(sa), _np16(Xa), M, K), "two streams")


def test_decode_sweep_full_output(pkg, oracle):
    """The benchmark layer's decode sweep checked on EVERY output (all 8192 rows), N = 1, 8 and 32: the library
    quantizes and packs on the GPU (the sampled-tile test above compares that stream with the oracle's), the
    oracle then computes the whole layer from those bytes in fp64."""
    name, M, K = workloads.FFN_65B
    _say("full output %s M=%d K=%d" % (name, M, K))
    W = workloads.make_weights(M, K, seed=0, device="cuda")
    packed, scales = pkg.fp6_quantize_pack(W)
    del W
    torch.cuda.synchronize()
    packed_h, scales_h = _np16(packed), _np16(scales)
    for N in (1, 8, 32):
        X = workloads.make_activations(N, K, seed=N, device="cuda")
        Y = pkg.fp6_linear(packed, scales, X, M, K)
        torch.cuda.synchronize()
        _say("  oracle on all rows, N=%d" % N)
        Y_ref = oracle.linear(packed_h, scales_h, _np16(X), M, K)
        worst = _check_linear(_np16(Y), Y_ref, "%s full N=%d" % (name, N))
        _say("    worst column ratio %.3g" % worst)
