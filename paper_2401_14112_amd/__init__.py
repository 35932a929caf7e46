"""MI355X-native W6A16 linear layer (FP6-LLM, arXiv 2401.14112).

The product is the C-ABI library built from csrc/ (see include/fp6.h); this package
is the thin Python binding over it.  PyTorch is used for device memory and streams
only - every step of the path runs in the library's HIP kernels.
"""
from .binding import (  # noqa: F401
    fp4_linear,
    fp3_linear,
    fp4_linear_workspace_bytes,
    fp3_linear_workspace_bytes,
    fp4_packed_bytes,
    fp3_packed_bytes,
    fp4_quantize_pack,
    fp3_quantize_pack,
    fp4_unpack,
    fp3_unpack,
    fp5_linear,
    fp5_linear_workspace_bytes,
    fp5_packed_bytes,
    fp5_quantize_pack,
    fp5_unpack,
    fp6g_linear,
    fp6g_quantize_pack,
    fp6g_unpack,
    fp6_layout_version,
    fp6_linear,
    fp6_linear_fused,
    fp6_linear_workspace_bytes,
    fp6_packed_bytes,
    fp6_quantize_pack,
    fp6_tuning_set_split_k,
    fp6_tuning_set_tile,
    fp6_unpack,
    fp6_workspace_init,
    fp16_linear,
    fp16_linear_workspace_bytes,
    library_path,
    load_library,
    Fp6Error,
)
