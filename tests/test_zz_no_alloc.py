"""fp6_linear_static, the entry point that allocates nothing (split-K state in a device array that is part of
the library), against fp6_linear on the same inputs: bit-identical outputs, on calls in a row with the later
ones smaller than the earlier ones, so that whatever an earlier call left in the shared array is in the way."""
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu


def _case(pkg, M, K, N, seed):
    W = workloads.make_weights(M, K, seed, device="cuda")
    packed, scales = pkg.fp6_quantize_pack(W)
    X = workloads.make_activations(N, K, seed + 1, device="cuda")
    return packed, scales, X


def test_static_entry_point_matches_fp6_linear_on_calls_in_a_row():
    import paper_2401_14112_amd as pkg

    # (M, K, N): streaming kernel with split-K at three token widths, the tiled kernel with split-K, then
    # smaller inputs again; the first is the largest
    shapes = [(2048, 8192, 40), (512, 4096, 8), (1024, 8192, 130), (256, 2048, 17), (512, 4096, 1)]
    cases = [_case(pkg, M, K, N, 11 * i) for i, (M, K, N) in enumerate(shapes)]
    expected = []
    for (M, K, N), (packed, scales, X) in zip(shapes, cases):
        assert pkg.fp6_linear_workspace_bytes(M, N, K) > 0, "the case is meant to use split-K"
        expected.append(pkg.fp6_linear(packed, scales, X, M, K))
    torch.cuda.synchronize()
    outs = [torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda") for M, K, N in shapes]
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for rounds in range(2):      # the second round starts from what the first left behind
        for (M, K, N), (packed, scales, X), out in zip(shapes, cases, outs):
            pkg.fp6_linear_static(packed, scales, X, M, K, out)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for (M, K, N), out, ref in zip(shapes, outs, expected):
        assert torch.equal(out.view(torch.int16), ref.view(torch.int16)), (M, K, N)


def test_static_entry_point_against_the_oracle():
    import numpy as np

    import paper_2401_14112_amd as pkg
    from oracle import fp6_oracle as oracle

    M, K = 512, 4096
    for N in (24, 3):     # two calls in a row, the second smaller
        W = workloads.make_weights(M, K, 5)
        X = workloads.make_activations(N, K, 6)
        packed, scales = pkg.fp6_quantize_pack(W.cuda())
        out = torch.empty((N, M), dtype=torch.float16, device="cuda")
        pkg.fp6_linear_static(packed, scales, X.cuda(), M, K, out)
        torch.cuda.synchronize()
        ref = oracle.linear(packed.cpu().numpy(), scales.cpu().numpy(), X.numpy(), M, K)
        err = np.abs(out.cpu().numpy().astype(np.float64) - ref).max(axis=1)
        assert (err <= 5e-3 * np.abs(ref).max(axis=1)).all()


def test_static_entry_point_refuses_what_does_not_fit():
    import paper_2401_14112_amd as pkg

    # the automatic plans never need more than the array holds; a forced split-K factor does
    M, K, N = 8192, 22016, 512
    packed = torch.empty(pkg.fp6_packed_bytes(M, K), dtype=torch.uint8, device="cuda")
    scales = torch.empty(M, dtype=torch.float16, device="cuda")
    X = torch.empty((N, K), dtype=torch.float16, device="cuda")
    out = torch.empty((N, M), dtype=torch.float16, device="cuda")
    pkg.fp6_tuning_set_split_k(4)
    try:
        assert pkg.fp6_linear_workspace_bytes(M, N, K) > (32 << 20) + (64 << 10)
        with pytest.raises(pkg.Fp6Error, match="WORKSPACE"):
            pkg.fp6_linear_static(packed, scales, X, M, K, out)
    finally:
        pkg.fp6_tuning_set_split_k(0)
