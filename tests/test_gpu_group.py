"""GPU parity tests of the group-wise-scale calls (fp6g_*), through the C-ABI binding, against the CPU oracle.

pack / unpack bit for bit; the GEMM within max_m |Y_gpu - Y_ref| <= 5e-3 * max_m |Y_ref| per output column.
"""
import numpy as np
import pytest
import torch

import workloads
from gpu_checks import check_linear as _check_linear
from packed_rows import row_tiles_of

pytestmark = pytest.mark.gpu

GROUP = 128


@pytest.fixture(scope="module")
def pkg():
    import paper_2401_14112_amd as p

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    p.load_library()
    return p


@pytest.fixture(scope="module")
def og():
    from oracle import fp6g_oracle
    return fp6g_oracle


def _say(msg):
    print(msg, flush=True)


def _np(t):
    return t.detach().cpu().numpy()


def _uneven_weights(M, K, seed, huge=True):
    """Weights whose column groups have very different ranges, plus zero groups and signed zeros."""
    W = workloads.make_weights(M, K, seed).numpy().copy()
    rng = np.random.default_rng(seed)
    factors = rng.choice([0.25, 1.0, 4.0, 16.0], size=(M, K // GROUP)).astype(np.float16)
    W = (W.reshape(M, K // GROUP, GROUP) * factors[:, :, None]).reshape(M, K).astype(np.float16)
    W[1, 0:GROUP] = 0
    W[1, 5] = -0.0
    W[2, GROUP:2 * GROUP] = np.float16(2.0 ** -24)      # scale rounds to zero
    if huge:
        W[3, 0] = np.float16(65504.0)                   # (its outputs overflow fp16: pack / unpack tests only)
    return W


@pytest.mark.parametrize("M,K,seed", [(256, 512, 0), (16, 256, 1), (80, 1280, 2)])
def test_quantize_pack_and_unpack_bit_exact(pkg, og, M, K, seed):
    _say("fp6g quantize_pack M=%d K=%d" % (M, K))
    W = _uneven_weights(M, K, seed)
    packed, scales = pkg.fp6g_quantize_pack(torch.from_numpy(W).cuda(), GROUP)
    back = pkg.fp6g_unpack(packed, scales, M, K, GROUP)
    torch.cuda.synchronize()
    ref_packed, ref_scales = og.quantize_pack(W, GROUP)
    assert scales.shape == (M, K // GROUP)
    assert np.array_equal(_np(scales).view(np.uint16), ref_scales.view(np.uint16))
    assert np.array_equal(_np(packed), ref_packed)
    assert np.array_equal(_np(back).view(np.uint16), og.unpack(ref_packed, ref_scales, M, K, GROUP).view(np.uint16))


def test_unsupported_group_is_refused(pkg):
    W = workloads.make_weights(16, 256, 0).cuda()
    with pytest.raises(pkg.Fp6Error):
        pkg.fp6g_quantize_pack(W, 64)


def _linear_case(pkg, og, M, K, N, seed, split=0):
    W = _uneven_weights(M, K, seed, huge=False)
    X = workloads.make_activations(N, K, seed)
    packed, scales = og.quantize_pack(W, GROUP)
    pkg.fp6_tuning_set_split_k(split)
    try:
        Y = pkg.fp6g_linear(torch.from_numpy(packed).cuda(), torch.from_numpy(scales).cuda(), X.cuda(), M, K, GROUP)
        torch.cuda.synchronize()
    finally:
        pkg.fp6_tuning_set_split_k(0)
    return _np(Y), og.linear(packed, scales, X.numpy(), M, K, GROUP)


@pytest.mark.parametrize("N", [1, 3, 16, 17, 32, 33, 64, 70, 130, 257])
def test_linear_token_counts(pkg, og, N):
    M, K = 80, 1280
    _say("fp6g linear M=%d K=%d N=%d" % (M, K, N))
    Y, Y_ref = _linear_case(pkg, og, M, K, N, seed=N)
    worst = _check_linear(Y, Y_ref, "N=%d" % N)
    assert worst < 3e-3


@pytest.mark.parametrize("split", [1, 2, 3, 5])
@pytest.mark.parametrize("N", [5, 48, 100])
def test_linear_split_k(pkg, og, split, N):
    M, K = 144, 2816
    _say("fp6g linear split-K S=%d N=%d" % (split, N))
    Y, Y_ref = _linear_case(pkg, og, M, K, N, seed=split, split=split)
    _check_linear(Y, Y_ref, "split=%d" % split)


def test_full_size_layer_sampled(pkg, og):
    name, M, K = workloads.FFN_65B
    _say("fp6g full-size %s M=%d K=%d" % (name, M, K))
    W = workloads.make_weights(M, K, seed=0, device="cuda")
    packed, scales = pkg.fp6g_quantize_pack(W, GROUP)
    torch.cuda.synchronize()
    rng = np.random.default_rng(1)
    tiles = np.array(sorted(set([0, M // 16 - 1]) | set(int(t) for t in rng.choice(M // 16, size=10, replace=False))))
    rows = (tiles[:, None] * 16 + np.arange(16)[None, :]).ravel()
    ref_packed, ref_scales = og.quantize_pack(_np(W[torch.from_numpy(rows).cuda()]), GROUP)
    got_packed = row_tiles_of(packed, M, K, tiles, 3072)
    assert np.array_equal(_np(scales)[rows].view(np.uint16), ref_scales.view(np.uint16))
    assert np.array_equal(got_packed, ref_packed)
    del W
    for N in (1, 16, 32, 512):
        _say("  fp6g linear N=%d" % N)
        X = workloads.make_activations(N, K, seed=N, device="cuda")
        Y = pkg.fp6g_linear(packed, scales, X, M, K, GROUP)
        torch.cuda.synchronize()
        Y_ref = og.linear(ref_packed, ref_scales, _np(X), len(rows), K, GROUP)
        _check_linear(_np(Y)[:, rows], Y_ref, "%s N=%d" % (name, N))
        outs = [pkg.fp6g_linear(packed, scales, X, M, K, GROUP) for _ in range(2)]
        torch.cuda.synchronize()
        assert torch.equal(outs[0].view(torch.int16), Y.view(torch.int16)) and torch.equal(outs[1].view(torch.int16), Y.view(torch.int16))
