"""ctypes binding of libfp6_mi355x.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/fp6.h).  Tensors
are torch CUDA tensors; outputs and workspaces are allocated here with torch when the
caller does not pass them.  There is no CPU fallback: if the library is missing and
cannot be built, or a tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path
from typing import Optional, Tuple

import torch

from . import build as _build

_lib = None


class Fp6Error(RuntimeError):
    pass


def library_path() -> Path:
    return _build.LIB


def load_library():
    """Load the built library; build it first only if no built library exists.  A library older than one of
    its sources is loaded as it is, with a warning: building is a step of its own (__graft_entry__.build()),
    never a side effect of a test or a benchmark run."""
    global _lib
    if _lib is not None:
        return _lib
    if not _build.LIB.exists():
        _build.build_library()
    elif _build.is_stale():
        import warnings

        warnings.warn("%s is older than its sources: rebuild with `python -m paper_2401_14112_amd.build`" % _build.LIB)
    L = ctypes.CDLL(str(_build.LIB))
    i64, vp, sz, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    L.fp6_status_str.restype = ctypes.c_char_p
    L.fp6_status_str.argtypes = [ci]
    L.fp6_layout_version.restype = ci
    L.fp6_layout_version.argtypes = []
    L.fp6_packed_bytes.restype = sz
    L.fp6_packed_bytes.argtypes = [i64, i64]
    L.fp6_linear_workspace_bytes.restype = sz
    L.fp6_linear_workspace_bytes.argtypes = [i64, i64, i64]
    L.fp16_linear_workspace_bytes.restype = sz
    L.fp16_linear_workspace_bytes.argtypes = [i64, i64, i64]
    L.fp6_workspace_init.restype = ci
    L.fp6_workspace_init.argtypes = [vp, sz, vp]
    L.fp6_quantize_pack.restype = ci
    L.fp6_quantize_pack.argtypes = [vp, i64, i64, vp, vp, vp]
    L.fp6_unpack.restype = ci
    L.fp6_unpack.argtypes = [vp, vp, i64, i64, vp, vp]
    L.fp6_linear.restype = ci
    L.fp6_linear.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, sz, vp]
    L.fp6_linear_static.restype = ci
    L.fp6_linear_static.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp]
    L.fp6_linear_fused.restype = ci
    L.fp6_linear_fused.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, vp, ci, vp, sz, vp]
    for _name in ("fp5_linear_fused", "fp4_linear_fused", "fp3_linear_fused"):
        getattr(L, _name).restype = ci
        getattr(L, _name).argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, vp, ci, vp, sz, vp]
    L.fp6g_linear_fused.restype = ci
    L.fp6g_linear_fused.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, vp, vp, ci, vp, sz, vp]
    L.fp6_probe_read.restype = ci
    L.fp6_probe_read.argtypes = [vp, sz, vp, vp]
    L.fp6_probe_read_bytes.restype = sz
    L.fp6_probe_read_bytes.argtypes = [sz]
    L.fp6_probe_mfma.restype = ci
    L.fp6_probe_mfma.argtypes = [i64, vp, vp]
    L.fp6_probe_mfma_sink_bytes.restype = sz
    L.fp6_probe_mfma_sink_bytes.argtypes = []
    L.fp16_linear.restype = ci
    L.fp16_linear.argtypes = [vp, vp, vp, i64, i64, i64, vp, sz, vp]
    L.fp5_packed_bytes.restype = sz
    L.fp5_packed_bytes.argtypes = [i64, i64]
    L.fp5_linear_workspace_bytes.restype = sz
    L.fp5_linear_workspace_bytes.argtypes = [i64, i64, i64]
    L.fp5_quantize_pack.restype = ci
    L.fp5_quantize_pack.argtypes = [vp, i64, i64, vp, vp, vp]
    L.fp5_unpack.restype = ci
    L.fp5_unpack.argtypes = [vp, vp, i64, i64, vp, vp]
    L.fp5_linear.restype = ci
    L.fp5_linear.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, sz, vp]
    L.fp4_packed_bytes.restype = sz
    L.fp4_packed_bytes.argtypes = [i64, i64]
    L.fp4_linear_workspace_bytes.restype = sz
    L.fp4_linear_workspace_bytes.argtypes = [i64, i64, i64]
    L.fp4_quantize_pack.restype = ci
    L.fp4_quantize_pack.argtypes = [vp, i64, i64, vp, vp, vp]
    L.fp4_unpack.restype = ci
    L.fp4_unpack.argtypes = [vp, vp, i64, i64, vp, vp]
    L.fp4_linear.restype = ci
    L.fp4_linear.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, sz, vp]
    L.fp3_packed_bytes.restype = sz
    L.fp3_packed_bytes.argtypes = [i64, i64]
    L.fp3_linear_workspace_bytes.restype = sz
    L.fp3_linear_workspace_bytes.argtypes = [i64, i64, i64]
    L.fp3_quantize_pack.restype = ci
    L.fp3_quantize_pack.argtypes = [vp, i64, i64, vp, vp, vp]
    L.fp3_unpack.restype = ci
    L.fp3_unpack.argtypes = [vp, vp, i64, i64, vp, vp]
    L.fp3_linear.restype = ci
    L.fp3_linear.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, sz, vp]
    L.fp6g_quantize_pack.restype = ci
    L.fp6g_quantize_pack.argtypes = [vp, i64, i64, i64, vp, vp, vp]
    L.fp6g_unpack.restype = ci
    L.fp6g_unpack.argtypes = [vp, vp, i64, i64, i64, vp, vp]
    L.fp6g_linear.restype = ci
    L.fp6g_linear.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, vp, sz, vp]
    L.fp6_tuning_set_split_k.restype = None
    L.fp6_tuning_set_split_k.argtypes = [ci]
    L.fp6_tuning_set_tile.restype = None
    L.fp6_tuning_set_tile.argtypes = [ci, ci]
    _lib = L
    return L


def _check(status: int):
    if status != 0:
        raise Fp6Error(load_library().fp6_status_str(status).decode())


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise Fp6Error("%s must be a CUDA tensor (there is no CPU path)" % name)
    if t.dtype != dtype:
        raise Fp6Error("%s must be %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise Fp6Error("%s must be contiguous" % name)
    return t


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def fp6_layout_version() -> int:
    return int(load_library().fp6_layout_version())


def fp6_packed_bytes(M: int, K: int) -> int:
    return int(load_library().fp6_packed_bytes(M, K))


def fp6_linear_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(load_library().fp6_linear_workspace_bytes(M, N, K))


def fp16_linear_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(load_library().fp16_linear_workspace_bytes(M, N, K))


def fp6_tuning_set_split_k(split_k: int) -> None:
    load_library().fp6_tuning_set_split_k(int(split_k))


def fp6_tuning_set_tile(block_rows: int, block_tokens: int) -> None:
    load_library().fp6_tuning_set_tile(int(block_rows), int(block_tokens))


def fp6_workspace_init(workspace: torch.Tensor) -> None:
    _dev(workspace, torch.uint8, "workspace")
    _check(load_library().fp6_workspace_init(workspace.data_ptr(), workspace.numel(), _stream()))


def _new_workspace(nbytes: int, device) -> Optional[torch.Tensor]:
    if nbytes == 0:
        return None
    return torch.zeros(nbytes, dtype=torch.uint8, device=device)


def _quantize_pack(prefix: str, W, packed, scales):
    L = load_library()
    _dev(W, torch.float16, "W")
    if W.dim() != 2:
        raise Fp6Error("W must be [M][K]")
    M, K = W.shape
    nbytes = getattr(L, prefix + "_packed_bytes")(M, K)
    if nbytes == 0:
        _check(2)
    if packed is None:
        packed = torch.empty(nbytes, dtype=torch.uint8, device=W.device)
    if scales is None:
        scales = torch.empty(M, dtype=torch.float16, device=W.device)
    _dev(packed, torch.uint8, "packed")
    _dev(scales, torch.float16, "scales")
    if packed.numel() != nbytes or scales.numel() != M:
        raise Fp6Error("packed/scales have the wrong size")
    _check(getattr(L, prefix + "_quantize_pack")(W.data_ptr(), M, K, packed.data_ptr(), scales.data_ptr(), _stream()))
    return packed, scales


def _unpack(prefix: str, packed, scales, M, K, out):
    L = load_library()
    _dev(packed, torch.uint8, "packed")
    _dev(scales, torch.float16, "scales")
    nbytes = getattr(L, prefix + "_packed_bytes")(M, K)
    if nbytes == 0:
        _check(2)
    if packed.numel() != nbytes or scales.numel() != M:
        raise Fp6Error("packed/scales do not match M, K")
    if out is None:
        out = torch.empty((M, K), dtype=torch.float16, device=packed.device)
    _dev(out, torch.float16, "out")
    if out.numel() != M * K:
        raise Fp6Error("out has the wrong size")
    _check(getattr(L, prefix + "_unpack")(packed.data_ptr(), scales.data_ptr(), M, K, out.data_ptr(), _stream()))
    return out


def _linear(prefix: str, packed, scales, X, M, K, out, workspace):
    L = load_library()
    _dev(packed, torch.uint8, "packed")
    _dev(scales, torch.float16, "scales")
    _dev(X, torch.float16, "X")
    if X.dim() != 2 or X.shape[1] != K:
        raise Fp6Error("X must be [N][K]")
    N = X.shape[0]
    nbytes = getattr(L, prefix + "_packed_bytes")(M, K)
    if nbytes == 0 or N == 0:
        _check(2)
    if packed.numel() != nbytes or scales.numel() != M:
        raise Fp6Error("packed/scales do not match M, K")
    if out is None:
        out = torch.empty((N, M), dtype=torch.float16, device=X.device)
    _dev(out, torch.float16, "out")
    if out.numel() != N * M:
        raise Fp6Error("out has the wrong size")
    if workspace is None:
        workspace = _new_workspace(getattr(L, prefix + "_linear_workspace_bytes")(M, N, K), X.device)
    ws_ptr, ws_len = (workspace.data_ptr(), workspace.numel()) if workspace is not None else (None, 0)
    _check(getattr(L, prefix + "_linear")(packed.data_ptr(), scales.data_ptr(), X.data_ptr(), out.data_ptr(), M, N, K,
                                          ws_ptr, ws_len, _stream()))
    return out


def fp6_quantize_pack(W: torch.Tensor, packed: Optional[torch.Tensor] = None,
                      scales: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """fp16 [M][K] -> (packed uint8 [3MK/4], scales fp16 [M])."""
    return _quantize_pack("fp6", W, packed, scales)


def fp6_unpack(packed: torch.Tensor, scales: torch.Tensor, M: int, K: int,
               out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """packed + scales -> fp16 [M][K]."""
    return _unpack("fp6", packed, scales, M, K, out)


def fp6_linear(packed: torch.Tensor, scales: torch.Tensor, X: torch.Tensor, M: int, K: int,
               out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y[N][M] = X[N][K] @ dequant(packed, scales)[M][K]^T  (fp16 in, fp16 out)."""
    return _linear("fp6", packed, scales, X, M, K, out, workspace)


def fp6_linear_static(packed: torch.Tensor, scales: torch.Tensor, X: torch.Tensor, M: int, K: int,
                      out: torch.Tensor) -> torch.Tensor:
    """fp6_linear on the library's own static split-K buffer: the entry point allocates nothing, and neither
    does this wrapper (`out` [N][M] is the caller's).  Calls that may overlap on one GPU race on that buffer."""
    L = load_library()
    _dev(packed, torch.uint8, "packed")
    _dev(scales, torch.float16, "scales")
    _dev(X, torch.float16, "X")
    _dev(out, torch.float16, "out")
    if X.dim() != 2 or X.shape[1] != K:
        raise Fp6Error("X must be [N][K]")
    N = X.shape[0]
    nbytes = L.fp6_packed_bytes(M, K)
    if nbytes == 0 or N == 0:
        _check(2)
    if packed.numel() != nbytes or scales.numel() != M or out.numel() != N * M:
        raise Fp6Error("packed/scales/out do not match M, N, K")
    _check(L.fp6_linear_static(packed.data_ptr(), scales.data_ptr(), X.data_ptr(), out.data_ptr(), M, N, K, _stream()))
    return out


def _linear_fused(prefix, packed, scales, X, M, K, bias, residual, gated, out, workspace, group=0):
    L = load_library()
    _dev(packed, torch.uint8, "packed")
    _dev(scales, torch.float16, "scales")
    _dev(X, torch.float16, "X")
    if X.dim() != 2 or X.shape[1] != K:
        raise Fp6Error("X must be [N][K]")
    N = X.shape[0]
    base = "fp6" if prefix == "fp6g" else prefix
    nbytes = getattr(L, base + "_packed_bytes")(M, K)
    if nbytes == 0 or N == 0 or (prefix == "fp6g" and (group <= 0 or K % group)):
        _check(2)
    n_scales = M * (K // group) if prefix == "fp6g" else M
    if packed.numel() != nbytes or scales.numel() != n_scales:
        raise Fp6Error("packed/scales do not match M, K")
    Mout = M // 2 if gated else M
    if bias is not None:
        _dev(bias, torch.float16, "bias")
        if bias.numel() != M:
            raise Fp6Error("bias must hold M values")
    if residual is not None:
        _dev(residual, torch.float16, "residual")
        if residual.numel() != N * Mout:
            raise Fp6Error("residual has the wrong size")
    if out is None:
        out = torch.empty((N, Mout), dtype=torch.float16, device=X.device)
    _dev(out, torch.float16, "out")
    if out.numel() != N * Mout:
        raise Fp6Error("out has the wrong size")
    if workspace is None:
        workspace = _new_workspace(getattr(L, base + "_linear_workspace_bytes")(M, N, K), X.device)
    ws_ptr, ws_len = (workspace.data_ptr(), workspace.numel()) if workspace is not None else (None, 0)
    head = (packed.data_ptr(), scales.data_ptr(), X.data_ptr(), out.data_ptr(), M, N, K)
    tail = (bias.data_ptr() if bias is not None else None, residual.data_ptr() if residual is not None else None,
            int(bool(gated)), ws_ptr, ws_len, _stream())
    fn = getattr(L, prefix + "_linear_fused")
    _check(fn(*head, group, *tail) if prefix == "fp6g" else fn(*head, *tail))
    return out


def fp6_linear_fused(packed: torch.Tensor, scales: torch.Tensor, X: torch.Tensor, M: int, K: int,
                     bias: Optional[torch.Tensor] = None, residual: Optional[torch.Tensor] = None,
                     gated: bool = False, out: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """fp6_linear followed, inside the kernel, by + bias[M], silu(row 2i) * row 2i+1 (gated) and + residual.

    Returns Y[N][Mout], Mout = M/2 when gated else M; residual has Y's shape and may be `out` itself."""
    return _linear_fused("fp6", packed, scales, X, M, K, bias, residual, gated, out, workspace)


def fp5_linear_fused(packed, scales, X, M, K, bias=None, residual=None, gated=False, out=None, workspace=None):
    return _linear_fused("fp5", packed, scales, X, M, K, bias, residual, gated, out, workspace)


def fp4_linear_fused(packed, scales, X, M, K, bias=None, residual=None, gated=False, out=None, workspace=None):
    return _linear_fused("fp4", packed, scales, X, M, K, bias, residual, gated, out, workspace)


def fp3_linear_fused(packed, scales, X, M, K, bias=None, residual=None, gated=False, out=None, workspace=None):
    return _linear_fused("fp3", packed, scales, X, M, K, bias, residual, gated, out, workspace)


def fp6g_linear_fused(packed, scales, X, M, K, group=128, bias=None, residual=None, gated=False, out=None,
                      workspace=None):
    return _linear_fused("fp6g", packed, scales, X, M, K, bias, residual, gated, out, workspace, group=group)


def fp5_packed_bytes(M: int, K: int) -> int:
    return int(load_library().fp5_packed_bytes(M, K))


def fp5_linear_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(load_library().fp5_linear_workspace_bytes(M, N, K))


def fp5_quantize_pack(W: torch.Tensor, packed: Optional[torch.Tensor] = None,
                      scales: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """fp16 [M][K] -> (packed uint8 [5MK/8], scales fp16 [M]), e2m2 codes."""
    return _quantize_pack("fp5", W, packed, scales)


def fp5_unpack(packed: torch.Tensor, scales: torch.Tensor, M: int, K: int,
               out: Optional[torch.Tensor] = None) -> torch.Tensor:
    return _unpack("fp5", packed, scales, M, K, out)


def fp5_linear(packed: torch.Tensor, scales: torch.Tensor, X: torch.Tensor, M: int, K: int,
               out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    return _linear("fp5", packed, scales, X, M, K, out, workspace)


def fp6g_quantize_pack(W: torch.Tensor, group: int = 128, packed: Optional[torch.Tensor] = None,
                       scales: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """fp16 [M][K] -> (packed uint8 [3MK/4], scales fp16 [M][K/group]): one scale per row and column group."""
    L = load_library()
    _dev(W, torch.float16, "W")
    if W.dim() != 2:
        raise Fp6Error("W must be [M][K]")
    M, K = W.shape
    nbytes = L.fp6_packed_bytes(M, K)
    if nbytes == 0 or group <= 0 or K % group:
        _check(2)
    if packed is None:
        packed = torch.empty(nbytes, dtype=torch.uint8, device=W.device)
    if scales is None:
        scales = torch.empty((M, K // group), dtype=torch.float16, device=W.device)
    _dev(packed, torch.uint8, "packed")
    _dev(scales, torch.float16, "scales")
    if packed.numel() != nbytes or scales.numel() != M * (K // group):
        raise Fp6Error("packed/scales have the wrong size")
    _check(L.fp6g_quantize_pack(W.data_ptr(), M, K, group, packed.data_ptr(), scales.data_ptr(), _stream()))
    return packed, scales


def fp6g_unpack(packed: torch.Tensor, scales: torch.Tensor, M: int, K: int, group: int = 128,
                out: Optional[torch.Tensor] = None) -> torch.Tensor:
    L = load_library()
    _dev(packed, torch.uint8, "packed")
    _dev(scales, torch.float16, "scales")
    nbytes = L.fp6_packed_bytes(M, K)
    if nbytes == 0 or group <= 0 or K % group:
        _check(2)
    if packed.numel() != nbytes or scales.numel() != M * (K // group):
        raise Fp6Error("packed/scales do not match M, K, group")
    if out is None:
        out = torch.empty((M, K), dtype=torch.float16, device=packed.device)
    _dev(out, torch.float16, "out")
    if out.numel() != M * K:
        raise Fp6Error("out has the wrong size")
    _check(L.fp6g_unpack(packed.data_ptr(), scales.data_ptr(), M, K, group, out.data_ptr(), _stream()))
    return out


def fp6g_linear(packed: torch.Tensor, scales: torch.Tensor, X: torch.Tensor, M: int, K: int, group: int = 128,
                out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    L = load_library()
    _dev(packed, torch.uint8, "packed")
    _dev(scales, torch.float16, "scales")
    _dev(X, torch.float16, "X")
    if X.dim() != 2 or X.shape[1] != K:
        raise Fp6Error("X must be [N][K]")
    N = X.shape[0]
    nbytes = L.fp6_packed_bytes(M, K)
    if nbytes == 0 or N == 0 or group <= 0 or K % group:
        _check(2)
    if packed.numel() != nbytes or scales.numel() != M * (K // group):
        raise Fp6Error("packed/scales do not match M, K, group")
    if out is None:
        out = torch.empty((N, M), dtype=torch.float16, device=X.device)
    _dev(out, torch.float16, "out")
    if out.numel() != N * M:
        raise Fp6Error("out has the wrong size")
    if workspace is None:
        workspace = _new_workspace(L.fp6_linear_workspace_bytes(M, N, K), X.device)
    ws_ptr, ws_len = (workspace.data_ptr(), workspace.numel()) if workspace is not None else (None, 0)
    _check(L.fp6g_linear(packed.data_ptr(), scales.data_ptr(), X.data_ptr(), out.data_ptr(), M, N, K, group,
                         ws_ptr, ws_len, _stream()))
    return out


def fp4_packed_bytes(M: int, K: int) -> int:
    return int(load_library().fp4_packed_bytes(M, K))


def fp4_linear_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(load_library().fp4_linear_workspace_bytes(M, N, K))


def fp4_quantize_pack(W: torch.Tensor, packed: Optional[torch.Tensor] = None,
                      scales: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """fp16 [M][K] -> (packed uint8 [MK/2], scales fp16 [M]), e2m1 codes."""
    return _quantize_pack("fp4", W, packed, scales)


def fp4_unpack(packed: torch.Tensor, scales: torch.Tensor, M: int, K: int,
               out: Optional[torch.Tensor] = None) -> torch.Tensor:
    return _unpack("fp4", packed, scales, M, K, out)


def fp4_linear(packed: torch.Tensor, scales: torch.Tensor, X: torch.Tensor, M: int, K: int,
               out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    return _linear("fp4", packed, scales, X, M, K, out, workspace)


def fp3_packed_bytes(M: int, K: int) -> int:
    return int(load_library().fp3_packed_bytes(M, K))


def fp3_linear_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(load_library().fp3_linear_workspace_bytes(M, N, K))


def fp3_quantize_pack(W: torch.Tensor, packed: Optional[torch.Tensor] = None,
                      scales: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """fp16 [M][K] -> (packed uint8 [3MK/8], scales fp16 [M]), e2m0 codes."""
    return _quantize_pack("fp3", W, packed, scales)


def fp3_unpack(packed: torch.Tensor, scales: torch.Tensor, M: int, K: int,
               out: Optional[torch.Tensor] = None) -> torch.Tensor:
    return _unpack("fp3", packed, scales, M, K, out)


def fp3_linear(packed: torch.Tensor, scales: torch.Tensor, X: torch.Tensor, M: int, K: int,
               out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    return _linear("fp3", packed, scales, X, M, K, out, workspace)


def fp16_linear(W: torch.Tensor, X: torch.Tensor, out: Optional[torch.Tensor] = None,
                workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y[N][M] = X[N][K] @ W[M][K]^T with the library's own fp16-weight kernel."""
    L = load_library()
    _dev(W, torch.float16, "W")
    _dev(X, torch.float16, "X")
    if W.dim() != 2 or X.dim() != 2 or X.shape[1] != W.shape[1]:
        raise Fp6Error("W must be [M][K] and X [N][K]")
    M, K = W.shape
    N = X.shape[0]
    if L.fp6_packed_bytes(M, K) == 0 or N == 0:
        _check(2)
    if out is None:
        out = torch.empty((N, M), dtype=torch.float16, device=X.device)
    _dev(out, torch.float16, "out")
    if workspace is None:
        workspace = _new_workspace(L.fp16_linear_workspace_bytes(M, N, K), X.device)
    ws_ptr, ws_len = (workspace.data_ptr(), workspace.numel()) if workspace is not None else (None, 0)
    _check(L.fp16_linear(W.data_ptr(), X.data_ptr(), out.data_ptr(), M, N, K, ws_ptr, ws_len, _stream()))
    return out


def fp6_probe_read(buffer: torch.Tensor, sink: Optional[torch.Tensor] = None) -> int:
    """Stream `buffer` once with the weight path's loads (diagnostic); returns the bytes actually read.
    sink (int32 [1024], device) receives, per wave w, the XOR of the 32-bit words of the 8 KB pieces w, 1024 + w, ..."""
    L = load_library()
    _dev(buffer, torch.uint8, "buffer")
    if sink is None:
        sink = torch.empty(1024, dtype=torch.int32, device=buffer.device)
    _dev(sink, torch.int32, "sink")
    if sink.numel() < 1024:
        raise Fp6Error("sink too small")
    _check(L.fp6_probe_read(buffer.data_ptr(), buffer.numel(), sink.data_ptr(), _stream()))
    return int(L.fp6_probe_read_bytes(buffer.numel()))


def fp6_probe_mfma(iters: int, sink: Optional[torch.Tensor] = None) -> float:
    """Issue iters x 4 matrix instructions (32x32x16, fp16) per wave on 4096 waves (diagnostic); returns the flop count."""
    L = load_library()
    if sink is None:
        sink = torch.empty(L.fp6_probe_mfma_sink_bytes(), dtype=torch.uint8, device="cuda")
    _dev(sink, torch.uint8, "sink")
    if sink.numel() < L.fp6_probe_mfma_sink_bytes():
        raise Fp6Error("sink too small")
    _check(L.fp6_probe_mfma(int(iters), sink.data_ptr(), _stream()))
    return 4096.0 * iters * 4 * 32768.0
