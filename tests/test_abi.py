"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
answers the size queries, and rejects bad arguments on the host before launching anything.
No compute call is made here (no GPU needed)."""
import ctypes
import glob
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2401_14112_amd as pkg

    return pkg.load_library()


def _declared_functions():
    text = ""
    for path in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        with open(path) as f:
            text += f.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(fp6g?_\w+|fp5_\w+|fp4_\w+|fp3_\w+|fp16_\w+)\s*\(", text)
    return sorted(set(names))


def test_exports_every_declared_symbol(lib):
    names = _declared_functions()
    for expected in ("fp6_quantize_pack", "fp6_unpack", "fp6_linear", "fp16_linear", "fp6_packed_bytes",
                     "fp6_linear_workspace_bytes", "fp6_workspace_init", "fp6_status_str", "fp6_layout_version",
                     "fp16_linear_workspace_bytes", "fp6_tuning_set_split_k", "fp6_tuning_set_tile",
                     "fp5_quantize_pack", "fp5_unpack", "fp5_linear", "fp5_packed_bytes", "fp5_linear_workspace_bytes",
                     "fp4_quantize_pack", "fp4_unpack", "fp4_linear", "fp4_packed_bytes", "fp4_linear_workspace_bytes",
                     "fp6g_quantize_pack", "fp6g_unpack", "fp6g_linear"):
        assert expected in names
    for n in names:
        assert hasattr(lib, n), "library does not export %s" % n


def test_binding_has_the_same_names():
    import paper_2401_14112_amd as pkg

    for n in ("fp6_quantize_pack", "fp6_unpack", "fp6_linear", "fp16_linear", "fp6_packed_bytes",
              "fp6_linear_workspace_bytes", "fp6_workspace_init", "fp6_layout_version",
              "fp5_quantize_pack", "fp5_unpack", "fp5_linear", "fp5_packed_bytes", "fp5_linear_workspace_bytes"):
        assert callable(getattr(pkg, n))


def test_size_queries(lib):
    assert lib.fp6_layout_version() >= 1
    assert lib.fp6_packed_bytes(8192, 22016) == 135266304          # 3*M*K/4
    assert lib.fp6_packed_bytes(256, 512) == 98304
    assert lib.fp6_packed_bytes(16, 256) == 3072
    # packed weights are addressed with 32-bit offsets: (K/256 + 64) * (M/16) * 3072 < 2^31, at every width
    assert lib.fp6_packed_bytes(32768, 49152) == 3 * 32768 * 49152 // 4
    assert lib.fp6_packed_bytes(65536, 65536) == 0 and lib.fp3_packed_bytes(65536, 65536) == 0
    assert lib.fp6_linear_workspace_bytes(65536, 1, 65536) == 0
    assert lib.fp5_packed_bytes(16, 256) == 2560 and lib.fp5_packed_bytes(8192, 22016) == 112721920
    assert lib.fp5_packed_bytes(15, 256) == 0
    assert lib.fp4_packed_bytes(16, 256) == 2048 and lib.fp4_packed_bytes(16, 128) == 0
    assert lib.fp6_packed_bytes(15, 256) == 0 and lib.fp6_packed_bytes(16, 128) == 0
    assert lib.fp6_packed_bytes(0, 256) == 0 and lib.fp6_packed_bytes(-16, 256) == 0
    assert lib.fp3_packed_bytes(16, 256) == 3072 and lib.fp3_packed_bytes(16, 512) == 3072 and lib.fp3_packed_bytes(8192, 22016) == 67633152
    # a token count whose activations exceed 2 GiB is cut into several launches: the query still answers
    assert lib.fp6_linear_workspace_bytes(32, 4194476, 256) % 16 == 0
    assert lib.fp6_linear_workspace_bytes(8192, 200000, 22016) <= 256 * 1024 * 1024
    for (M, N, K) in [(8192, 1, 22016), (8192, 32, 22016), (256, 8, 512), (22016, 16, 8192)]:
        b = lib.fp6_linear_workspace_bytes(M, N, K)
        assert b % 16 == 0
        assert b <= 64 * 1024 * 1024


def test_bad_arguments_are_rejected_on_the_host(lib):
    OK, NULL, SHAPE, WS, ALIGN = 0, 1, 2, 3, 4
    p = ctypes.c_void_p(0x10000)          # never dereferenced: every call below fails its checks first
    odd = ctypes.c_void_p(0x10008)
    null = ctypes.c_void_p(0)
    assert lib.fp6_quantize_pack(null, 16, 256, p, p, null) == NULL
    assert lib.fp6_quantize_pack(p, 16, 100, p, p, null) == SHAPE
    assert lib.fp6_quantize_pack(p, 10, 256, p, p, null) == SHAPE
    assert lib.fp6_quantize_pack(p, 16, 256, odd, p, null) == ALIGN
    assert lib.fp6_unpack(p, null, 16, 256, p, null) == NULL
    assert lib.fp6_unpack(p, p, 0, 256, p, null) == SHAPE
    assert lib.fp6_unpack(odd, p, 16, 256, p, null) == ALIGN
    assert lib.fp6_linear(p, p, p, null, 16, 1, 256, null, 0, null) == NULL
    assert lib.fp6_linear(p, p, p, p, 16, 0, 256, null, 0, null) == SHAPE
    assert lib.fp6_linear(p, p, p, p, 16, 1, 255, null, 0, null) == SHAPE
    assert lib.fp6_linear(p, p, odd, p, 16, 1, 256, null, 0, null) == ALIGN
    assert lib.fp6_linear_fused(p, p, p, null, 16, 1, 256, null, null, 0, null, 0, null) == NULL
    assert lib.fp6_linear_fused(p, p, p, p, 16, 1, 256, odd, null, 0, null, 0, null) == ALIGN
    assert lib.fp6_linear_fused(p, p, p, p, 16, 1, 256, null, odd, 1, null, 0, null) == ALIGN
    assert lib.fp6_linear_fused(p, p, p, p, 16, 0, 256, null, null, 1, null, 0, null) == SHAPE
    assert lib.fp3_linear(p, p, p, p, 16, 1, 128, null, 0, null) == SHAPE
    assert lib.fp6g_linear(p, p, p, p, 16, 1, 256, 64, null, 0, null) == SHAPE       # only groups of 128 columns
    assert lib.fp16_linear(null, p, p, 16, 1, 256, null, 0, null) == NULL
    assert lib.fp16_linear(p, p, p, 24, 1, 256, null, 0, null) == SHAPE
    # 32-bit byte offsets into the activations and into fp16 weight rows: K stops below 2^24
    big_k = 1 << 24
    assert lib.fp6_packed_bytes(16, big_k) == 0 and lib.fp6_packed_bytes(16, big_k - 256) == 3 * 16 * (big_k - 256) // 4
    assert lib.fp6_linear(p, p, p, p, 16, 1, big_k, null, 0, null) == SHAPE
    assert lib.fp16_linear(p, p, p, 16, 1, big_k, null, 0, null) == SHAPE
    assert lib.fp16_linear(p, p, p, 16, 128, big_k, null, 0, null) == SHAPE
    assert lib.fp16_linear_workspace_bytes(16, 1, big_k) == 0
    # the entry point that allocates nothing refuses bad arguments, and shapes that do not fit its array, on
    # the host as well (a forced split-K factor is the only way past the array's size)
    assert lib.fp6_linear_static(p, p, p, null, 16, 1, 256, null) == NULL
    assert lib.fp6_linear_static(p, p, p, p, 16, 0, 256, null) == SHAPE
    assert lib.fp6_linear_static(p, odd, p, p, 16, 1, 256, null) == ALIGN
    lib.fp6_tuning_set_split_k(4)
    try:
        assert lib.fp6_linear_workspace_bytes(8192, 512, 22016) > (32 << 20) + (64 << 10)
        assert lib.fp6_linear_static(p, p, p, p, 8192, 512, 22016, null) == WS
    finally:
        lib.fp6_tuning_set_split_k(0)
    # a shape that needs split-K partial sums refuses to run without a workspace
    M, N, K = 8192, 8, 22016
    need = lib.fp6_linear_workspace_bytes(M, N, K)
    assert need > 0
    assert lib.fp6_linear(p, p, p, p, M, N, K, null, 0, null) == WS
    assert lib.fp6_linear(p, p, p, p, M, N, K, p, need - 16, null) == WS
    assert lib.fp6_linear(p, p, p, p, M, N, K, odd, need, null) == ALIGN
    assert lib.fp6_workspace_init(null, 0, null) == OK
    assert lib.fp6_workspace_init(null, 64, null) == NULL
    assert lib.fp6_workspace_init(odd, 64, null) == ALIGN
    for code in range(0, 7):
        assert len(lib.fp6_status_str(code)) > 0


def test_binding_refuses_cpu_tensors():
    import torch

    import paper_2401_14112_amd as pkg

    W = torch.zeros((16, 256), dtype=torch.float16)
    with pytest.raises(pkg.Fp6Error):
        pkg.fp6_quantize_pack(W)
    with pytest.raises(pkg.Fp6Error):
        pkg.fp6_linear(torch.zeros(3072, dtype=torch.uint8), torch.zeros(16, dtype=torch.float16),
                       torch.zeros((1, 256), dtype=torch.float16), 16, 256)
