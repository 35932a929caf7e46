"""GPU parity tests of fp6_linear_fused (bias, silu(gate) * up, residual in the kernel's last step) against
the CPU oracle, through the C-ABI binding.  Same bound as the plain layer: for every token column n,
max_o |Y_gpu - Y_ref| <= 5e-3 * max_o |Y_ref| (Y_ref in fp64, no intermediate rounding).
"""
import numpy as np
import pytest
import torch

import workloads
from gpu_checks import check_linear as _check
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


def _np(t):
    return t.detach().cpu().numpy()


MODES = {
    "bias": dict(bias=True, residual=False, gated=False),
    "residual": dict(bias=False, residual=True, gated=False),
    "gated": dict(bias=False, residual=False, gated=True),
    "all": dict(bias=True, residual=True, gated=True),
    "bias_residual": dict(bias=True, residual=True, gated=False),
}


def _inputs(M, K, N, seed, mode):
    Mout = M // 2 if mode["gated"] else M
    W = workloads.make_weights(M, K, seed).numpy()
    X = workloads.make_activations(N, K, seed)
    # bias and residual of the size of the products (std ~ 0.02 * sqrt(K)), so a dropped or misplaced one shows
    amp = 0.02 * np.sqrt(K)
    bias = (workloads.make_activations(1, M, seed + 100)[0] * amp).to(torch.float16) if mode["bias"] else None
    R = (workloads.make_activations(N, Mout, seed + 200) * amp).to(torch.float16) if mode["residual"] else None
    return W, X, bias, R


def _case(pkg, oracle, M, K, N, seed, mode, split=0, tile=None, in_place=False):
    W, X, bias, R = _inputs(M, K, N, seed, mode)
    packed, scales = oracle.quantize_pack(W)
    Y_ref = oracle.linear_fused(packed, scales, X.numpy(), M, K, bias=None if bias is None else bias.numpy(),
                                residual=None if R is None else R.numpy(), gated=mode["gated"])
    pkg.fp6_tuning_set_split_k(split)
    if tile:
        pkg.fp6_tuning_set_tile(*tile)
    try:
        Rd = None if R is None else R.cuda()
        Y = pkg.fp6_linear_fused(torch.from_numpy(packed).cuda(), torch.from_numpy(scales).cuda(), X.cuda(), M, K,
                                 bias=None if bias is None else bias.cuda(), residual=Rd, gated=mode["gated"],
                                 out=Rd if in_place else None)
        torch.cuda.synchronize()
    finally:
        pkg.fp6_tuning_set_split_k(0)
        pkg.fp6_tuning_set_tile(0, 0)
    assert Y.shape == Y_ref.shape
    return _np(Y), Y_ref


@pytest.mark.parametrize("mode", sorted(MODES))
@pytest.mark.parametrize("N", [1, 5, 16, 17, 33, 64, 70, 130])
def test_fused_modes_and_token_counts(pkg, oracle, mode, N):
    M, K = 80, 1280          # 5 row tiles (ragged against the blocks), 5 k-tiles; N spans all kernels
    _say("fused %s M=%d K=%d N=%d" % (mode, M, K, N))
    Y, Y_ref = _case(pkg, oracle, M, K, N, seed=N, mode=MODES[mode])
    _check(Y, Y_ref, "%s N=%d" % (mode, N))


@pytest.mark.parametrize("split", [1, 3, 64])
@pytest.mark.parametrize("N", [5, 32, 96])
def test_fused_split_k(pkg, oracle, split, N):
    M, K = 144, 2816
    _say("fused all split-K S=%d N=%d" % (split, N))
    Y, Y_ref = _case(pkg, oracle, M, K, N, seed=split, mode=MODES["all"], split=split)
    _check(Y, Y_ref, "split=%d" % split)


@pytest.mark.parametrize("tile", [(128, 128), (128, 64), (256, 128), (256, 64)])
def test_fused_every_tile_shape(pkg, oracle, tile):
    M, K, N = 528, 768, 200       # ragged against 128- and 256-row blocks and against 64/128-token blocks
    _say("fused all tile=%s" % (tile,))
    Y, Y_ref = _case(pkg, oracle, M, K, N, seed=8, mode=MODES["all"], tile=tile)
    _check(Y, Y_ref, "tile=%s" % (tile,))


@pytest.mark.parametrize("mode", ["residual", "all"])
@pytest.mark.parametrize("N", [7, 100])
def test_fused_residual_in_place(pkg, oracle, mode, N):
    """The residual stream is updated in place: Y is the residual buffer itself."""
    M, K = 160, 1024
    _say("fused %s in place N=%d" % (mode, N))
    Y, Y_ref = _case(pkg, oracle, M, K, N, seed=N, mode=MODES[mode], in_place=True)
    _check(Y, Y_ref, "in place")


def test_fused_without_steps_equals_plain(pkg, oracle):
    M, K = 96, 1536
    W = workloads.make_weights(M, K, 4).cuda()
    packed, scales = pkg.fp6_quantize_pack(W)
    for N in (3, 48, 80):
        _say("fused with no step N=%d" % N)
        X = workloads.make_activations(N, K, N).cuda()
        a = pkg.fp6_linear(packed, scales, X, M, K)
        b = pkg.fp6_linear_fused(packed, scales, X, M, K)
        torch.cuda.synchronize()
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_fused_closed_form(pkg, oracle):
    """Products crafted to be exact (one weight of 1.0 or 2.0 per row, scale 1): the output is the fp16
    rounding of silu(g) * u + r up to the fp32 evaluation of the logistic function."""
    _say("fused closed form")
    M, K, N = 32, 256, 3
    codes = np.zeros((M, K), dtype=np.uint8)
    for i in range(M // 2):
        codes[2 * i, 2 * i] = 0b001100        # gate row: 1.0 at column 2i
        codes[2 * i + 1, 2 * i + 1] = 0b010000  # up row: 2.0 at column 2i+1
    rng = np.random.default_rng(3)
    g = rng.uniform(-6, 6, (N, M // 2)).astype(np.float16)
    g[0, :4] = [0.0, 1.0, -1.0, 12.0]
    u = rng.uniform(-3, 3, (N, M // 2)).astype(np.float16)
    X = np.zeros((N, K), dtype=np.float16)
    X[:, 0:M:2] = g
    X[:, 1:M:2] = u / 2
    u = (X[:, 1:M:2].astype(np.float64) * 2)
    R = rng.uniform(-1, 1, (N, M // 2)).astype(np.float16)
    Y = pkg.fp6_linear_fused(torch.from_numpy(oracle.pack(codes)).cuda(), torch.ones(M, dtype=torch.float16).cuda(),
                             torch.from_numpy(X).cuda(), M, K, residual=torch.from_numpy(R).cuda(), gated=True)
    torch.cuda.synchronize()
    gd = g.astype(np.float64)
    want = gd / (1 + np.exp(-gd)) * u + R.astype(np.float64)
    got = _np(Y).astype(np.float64)
    # one fp16 rounding (2^-11 relative) plus the fp32 logistic function
    assert np.all(np.abs(got - want) <= 2.0 ** -10 * np.abs(want) + 2.0 ** -24 + 1e-5 * np.abs(gd * u))
    assert got[0, 0] == float(R[0, 0])        # silu(0) * u = 0 exactly


def test_fused_rejects_misaligned_and_mismatched(pkg):
    M, K, N = 32, 256, 2
    packed = torch.zeros(pkg.fp6_packed_bytes(M, K), dtype=torch.uint8, device="cuda")
    scales = torch.ones(M, dtype=torch.float16, device="cuda")
    X = torch.zeros((N, K), dtype=torch.float16, device="cuda")
    buf = torch.zeros(M + 8, dtype=torch.float16, device="cuda")
    with pytest.raises(pkg.Fp6Error, match="ALIGN"):
        pkg.fp6_linear_fused(packed, scales, X, M, K, bias=buf[1:M + 1])
    with pytest.raises(pkg.Fp6Error, match="residual"):
        pkg.fp6_linear_fused(packed, scales, X, M, K, residual=torch.zeros((N, M), dtype=torch.float16, device="cuda"),
                             gated=True)
    with pytest.raises(pkg.Fp6Error, match="bias"):
        pkg.fp6_linear_fused(packed, scales, X, M, K, bias=buf[:M // 2], gated=True)


def _sampled_tiles(M, count, seed):
    n_tiles = M // 16
    rng = np.random.default_rng(seed)
    picks = set([0, n_tiles - 1])
    while len(picks) < min(count, n_tiles):
        picks.add(int(rng.integers(0, n_tiles)))
    return np.array(sorted(picks), dtype=np.int64)


@pytest.mark.parametrize("N", [1, 16, 32, 512])
def test_fused_full_size_decoder_projections(pkg, oracle, N):
    """The feed-forward block of a 70B-class decoder at its real sizes, in the launch configurations the
    benchmark times: gate and up interleaved row by row (M = 2 x 28672, K = 8192) with the gated step, then
    the down projection (M = 8192, K = 28672) adding to the residual in place.  Sampled row tiles against
    the oracle; weights are quantized on the GPU and the sampled tiles checked byte for byte first."""
    F, H = 28672, 8192
    _say("fused feed-forward block N=%d" % N)
    X = workloads.make_activations(N, H, seed=N, device="cuda")
    W = workloads.make_weights(2 * F, H, seed=21, device="cuda")
    packed, scales = pkg.fp6_quantize_pack(W)
    bias = (workloads.make_activations(1, 2 * F, seed=5, device="cuda")[0] * 0.5).to(torch.float16)
    torch.cuda.synchronize()
    tiles = _sampled_tiles(2 * F, 12, seed=N)
    rows = (tiles[:, None] * 16 + np.arange(16)[None, :]).ravel()
    out_rows = rows[::2] // 2
    ref_packed, ref_scales = oracle.quantize_pack(_np(W[torch.from_numpy(rows).cuda()]))
    got_packed = row_tiles_of(packed, 2 * F, H, tiles, 3072)
    assert np.array_equal(got_packed, ref_packed)
    assert np.array_equal(_np(scales)[rows].view(np.uint16), ref_scales.view(np.uint16))
    del W
    A = pkg.fp6_linear_fused(packed, scales, X, 2 * F, H, bias=bias, gated=True)
    torch.cuda.synchronize()
    assert A.shape == (N, F)
    ref = oracle.linear_fused(ref_packed, ref_scales, _np(X), len(rows), H, bias=_np(bias)[rows], gated=True)
    worst = _check(_np(A)[:, out_rows], ref, "gate/up N=%d" % N)
    _say("  gate/up worst column ratio %.3g" % worst)
    del packed, scales

    W2 = workloads.make_weights(H, F, seed=22, device="cuda")
    packed2, scales2 = pkg.fp6_quantize_pack(W2)
    torch.cuda.synchronize()
    tiles2 = _sampled_tiles(H, 6, seed=N + 1)
    rows2 = (tiles2[:, None] * 16 + np.arange(16)[None, :]).ravel()
    ref_packed2, ref_scales2 = oracle.quantize_pack(_np(W2[torch.from_numpy(rows2).cuda()]))
    del W2
    A = (A * 4).to(torch.float16)        # activations of order 1 for the second projection
    R = workloads.make_activations(N, H, seed=N + 9, device="cuda")
    R0 = _np(R).copy()
    pkg.fp6_linear_fused(packed2, scales2, A, H, F, residual=R, out=R)
    torch.cuda.synchronize()
    ref2 = oracle.linear_fused(ref_packed2, ref_scales2, _np(A), len(rows2), F, residual=R0[:, rows2])
    worst = _check(_np(R)[:, rows2], ref2, "down N=%d" % N)
    _say("  down + residual worst column ratio %.3g" % worst)


@pytest.mark.parametrize("fmt", ["fp5", "fp4", "fp3", "fp6g"])
@pytest.mark.parametrize("mode", ["all", "bias_residual"])
@pytest.mark.parametrize("N", [5, 40, 100])
def test_fused_other_formats(pkg, oracle, fmt, mode, N):
    """The same steps after the 5-, 4-, 3-bit layers and the layer with group-wise scales."""
    import importlib
    M, K = 96, 1536
    _say("fused %s %s N=%d" % (fmt, mode, N))
    m = MODES[mode]
    W, X, bias, R = _inputs(M, K, N, seed=N + len(fmt), mode=m)
    kw = dict(bias=None if bias is None else bias.cuda(), residual=None if R is None else R.cuda(), gated=m["gated"])
    okw = dict(bias=None if bias is None else bias.numpy(), residual=None if R is None else R.numpy(), gated=m["gated"])
    if fmt == "fp6g":
        from oracle import fp6g_oracle
        packed, scales = fp6g_oracle.quantize_pack(W, 128)
        Y_ref = oracle.linear_fused(packed, scales, X.numpy(), M, K, group=128, **okw)
        Y = pkg.fp6g_linear_fused(torch.from_numpy(packed).cuda(), torch.from_numpy(scales).cuda(), X.cuda(), M, K, 128, **kw)
    else:
        bits = int(fmt[2])
        from oracle import fpx_oracle
        o = fpx_oracle.BY_PREFIX[fmt] if fmt in fpx_oracle.BY_PREFIX else importlib.import_module("oracle.%s_oracle" % fmt)
        packed, scales = o.quantize_pack(W)
        Y_ref = oracle.linear_fused(packed, scales, X.numpy(), M, K, bits=bits, **okw)
        Y = getattr(pkg, fmt + "_linear_fused")(torch.from_numpy(packed).cuda(), torch.from_numpy(scales).cuda(), X.cuda(), M, K, **kw)
    torch.cuda.synchronize()
    assert Y.shape == Y_ref.shape
    _check(_np(Y), Y_ref, "%s %s N=%d" % (fmt, mode, N))
