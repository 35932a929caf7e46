"""Seeded synthetic inputs and the layer shapes of the benchmark configurations.

This module is shared by the CPU oracle's tests and by the HIP path's tests and
benchmark.  It holds none of the method's arithmetic: it only draws random
matrices and names shapes.  The real workloads of the paper (LLaMA / OPT linear
layers, Section 7.1) are trained weights that are not available; the stand-in is
W ~ N(0, 0.02) drawn in fp32 and cast once to fp16, X ~ N(0, 1) cast to fp16,
stored [N][K] (the column-major activation layout of Section 6).
"""
from __future__ import annotations

import torch

# (name, M = output features, K = input features)
TINY = ("tiny", 256, 512)
FFN_65B = ("llama65b_ffn_up", 8192, 22016)       # headline layer (Fig. 1 of the paper)
FFN_65B_DOWN = ("llama65b_ffn_down", 22016, 8192)
SET_70B = [
    ("70b_qkv", 10240, 8192),
    ("70b_o", 8192, 8192),
    ("70b_gate_up", 28672, 8192),
    ("70b_down", 8192, 28672),
]
# Decoder-block linear layers of the model families whose shapes the paper's kernel benchmark sweeps
# (Section 7.1: LLaMA-7b/13b/33b/65b, OPT-30b/66b/175b at batch 8, 16, 32): (hidden, feed-forward inner,
# gated).  Per block: QKV [3h][h], attention output [h][h], feed-forward in [f][h] (twice for the gated
# LLaMA form, stacked as [2f][h]) and out [h][f].  Architecture constants only; weights are synthetic.
MODEL_DIMS = [
    ("llama-7b", 4096, 11008, True),
    ("llama-13b", 5120, 13824, True),
    ("llama-33b", 6656, 17920, True),
    ("llama-65b", 8192, 22016, True),
    ("opt-30b", 7168, 28672, False),
    ("opt-66b", 9216, 36864, False),
    ("opt-175b", 12288, 49152, False),
]


def model_layers(hidden: int, inner: int, gated: bool):
    """(name, M, K) of the four linear layers of one decoder block."""
    return [("qkv", 3 * hidden, hidden), ("attn_out", hidden, hidden),
            ("ffn_in", (2 if gated else 1) * inner, hidden), ("ffn_out", hidden, inner)]


DECODE_N = [1, 2, 4, 8, 16, 32]
PREFILL_N = [64, 128, 256, 512]

W_STD = 0.02


def make_weights(M: int, K: int, seed: int = 0, device: str = "cpu") -> torch.Tensor:
    """fp16 [M][K]: N(0, 0.02) drawn in fp32 with a seeded generator, cast once."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    w = torch.empty((M, K), dtype=torch.float32, device=device)
    w.normal_(0.0, W_STD, generator=g)
    return w.to(torch.float16)


def make_activations(N: int, K: int, seed: int = 0, device: str = "cpu") -> torch.Tensor:
    """fp16 [N][K]: N(0, 1).  A different stream from the weights of the same seed."""
    g = torch.Generator(device=device)
    g.manual_seed(seed + 0x5EED)
    x = torch.empty((N, K), dtype=torch.float32, device=device)
    x.normal_(0.0, 1.0, generator=g)
    return x.to(torch.float16)


def make_codes(M: int, K: int, seed: int = 0) -> torch.Tensor:
    """uint8 [M][K] uniform over the 64 codes (layout tests)."""
    g = torch.Generator()
    g.manual_seed(seed)
    return torch.randint(0, 64, (M, K), dtype=torch.uint8, generator=g)
