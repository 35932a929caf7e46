"""Seeded random shapes through every width of the library against its oracle: row-tile counts that are odd,
prime or one (the tiles of a row tile are M/16 tiles apart in the packed stream), k-tile counts from 1 up,
token counts on both sides of every kernel switch, and forced split-K factors.  Pack and unpack bit for bit,
the linear layer within the column bound."""
import importlib

import numpy as np
import pytest
import torch

import workloads
from gpu_checks import check_linear

pytestmark = pytest.mark.gpu

WIDTHS = ("fp6", "fp5", "fp4", "fp3", "fp6g")


def _cases():
    rng = np.random.default_rng(20240114)
    cases = []
    for i in range(30):
        width = WIDTHS[i % len(WIDTHS)]
        M = 16 * int(rng.choice([1, 2, 3, 5, 7, 11, 13, 17, 23, 31, 37]))
        K = 256 * int(rng.choice([1, 2, 3, 4, 5, 7, 9, 12]))
        N = int(rng.choice([1, 2, 7, 15, 16, 17, 31, 32, 33, 63, 64, 65, 100, 129, 150]))
        split = int(rng.choice([0, 0, 1, 2, 3, 5]))
        cases.append((width, M, K, N, split, 1000 + i))
    return cases


@pytest.fixture(scope="module")
def pkg():
    import paper_2401_14112_amd as p

    p.load_library()
    return p


def _oracle(width):
    from oracle import fp6_oracle

    fp6_oracle.build()      # one C library serves every width
    from oracle import fpx_oracle

    return fpx_oracle.BY_PREFIX[width] if width in fpx_oracle.BY_PREFIX else importlib.import_module("oracle.%s_oracle" % width)


@pytest.mark.parametrize("width,M,K,N,split,seed", _cases())
def test_random_shape(pkg, width, M, K, N, split, seed):
    print("random shape %s M=%d K=%d N=%d split=%d seed=%d" % (width, M, K, N, split, seed), flush=True)
    o = _oracle(width)
    group = (128,) if width == "fp6g" else ()
    W = workloads.make_weights(M, K, seed)
    X = workloads.make_activations(N, K, seed + 1)
    packed, scales = getattr(pkg, width + "_quantize_pack")(W.cuda(), *group)
    torch.cuda.synchronize()
    ref_packed, ref_scales = o.quantize_pack(W.numpy(), *group)
    assert np.array_equal(packed.cpu().numpy(), ref_packed)
    assert np.array_equal(scales.cpu().numpy().view(np.uint16), ref_scales.view(np.uint16))
    Wd = getattr(pkg, width + "_unpack")(packed, scales, M, K, *group)
    torch.cuda.synchronize()
    assert np.array_equal(Wd.cpu().numpy().view(np.uint16), o.unpack(ref_packed, ref_scales, M, K, *group).view(np.uint16))
    pkg.fp6_tuning_set_split_k(split)
    try:
        Y = getattr(pkg, width + "_linear")(packed, scales, X.cuda(), M, K, *group)
        torch.cuda.synchronize()
    finally:
        pkg.fp6_tuning_set_split_k(0)
    Y_ref = o.linear(ref_packed, ref_scales, X.numpy(), M, K, *group)
    check_linear(Y.cpu().numpy(), Y_ref, "%s M=%d K=%d N=%d split=%d" % (width, M, K, N, split))
