"""Thin Python binding of libtbik (argument marshalling only).

Every function has the name of the C entry point it calls (``include/tbik.h``) and takes
``torch`` tensors that already live on the GPU: PyTorch provides device memory and the current
HIP stream, nothing else.  No arithmetic of the method happens in Python, and there is no CPU
fallback: if ``libtbik.so`` is missing the import of the library fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# TBIK_LIB_PATH points development runs at an alternative build of the same library.
LIB_PATH = os.environ.get("TBIK_LIB_PATH") or os.path.join(_HERE, "libtbik.so")

TBIK_F32, TBIK_BF16, TBIK_F16 = 0, 1, 2
TBIK_SUM, TBIK_MAX, TBIK_LOGSOFTMAX = 0, 1, 2
OK = 0

VARIANT_AUTO, VARIANT_REFERENCE, VARIANT_T128, VARIANT_T32, VARIANT_T64 = 0, 1, 2, 3, 4

# name -> (restype, argtypes); mirrors include/tbik.h
SIGNATURES = {
    "tbik_gemm": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int,
                            C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_gemm_shard_partials": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p,
                                           C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                           C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_tree_combine": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "tbik_rmsnorm": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_void_p]),
    "tbik_row_reduce": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int64,
                                  C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_row_reduce_static": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int64, C.c_void_p]),
    "tbik_gemm_mxfp4": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                  C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                  C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_gemm_shard_partials_mxfp4": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                                 C.c_void_p, C.c_int64, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                                 C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_gemm_reference_mxfp4": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                            C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_int,
                                            C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "tbik_gemm_mxfp4_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]),
    "tbik_gemm_mxfp8": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                  C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                  C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_gemm_shard_partials_mxfp8": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                                 C.c_void_p, C.c_int64, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                                 C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_gemm_reference_mxfp8": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                            C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_int,
                                            C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "tbik_gemm_mxfp8_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]),
    "tbik_gemm_mxfp6": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                  C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                  C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_gemm_shard_partials_mxfp6": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                                 C.c_void_p, C.c_int64, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                                 C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_gemm_reference_mxfp6": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                            C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_int,
                                            C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "tbik_gemm_mxfp6_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]),
    "tbik_tree_allreduce": (C.c_int, [C.c_void_p, C.c_int, C.c_int64, C.c_void_p]),
    "tbik_silu_mul": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int,
                                C.c_void_p]),
    "tbik_gemm_swiglu": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int,
                                   C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_gemm_swiglu_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]),
    "tbik_gemm_fp8": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int, C.c_int,
                                C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_gemm_shard_partials_fp8": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int,
                                               C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                               C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_gemm_reference_fp8": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64,
                                          C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "tbik_gemm_fp8_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]),
    "tbik_gemm_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]),
    "tbik_row_reduce_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int64, C.c_int]),
    "tbik_gemm_reference": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64,
                                      C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "tbik_gemm_f16": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int,
                                C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_gemm_shard_partials_f16": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p,
                                               C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                               C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_gemm_reference_f16": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64,
                                          C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "tbik_combine_residual_rmsnorm": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p,
                                                C.c_int, C.c_int, C.c_void_p]),
    "tbik_gemm_f32": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_gemm_shard_partials_f32": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p,
                                               C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                               C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_gemm_reference_f32": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64,
                                          C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "tbik_rmsnorm_f16": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_void_p]),
    "tbik_combine_residual_rmsnorm_f16": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p,
                                                    C.c_void_p, C.c_int, C.c_int, C.c_void_p]),
    "tbik_attention": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                 C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_int64,
                                 C.c_float, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_attention_f16": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                 C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_int64,
                                 C.c_float, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tbik_attention_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]),
    "tbik_set_gemm_variant": (C.c_int, [C.c_int]),
    "tbik_set_attention_variant": (C.c_int, [C.c_int]),
    "tbik_set_row_wait_limit": (C.c_int, [C.c_int]),
    "tbik_variant_name": (C.c_char_p, [C.c_int]),
    "tbik_status_string": (C.c_char_p, [C.c_int]),
    "tbik_last_hip_error": (C.c_int, []),
    "tbik_version": (C.c_char_p, []),
}

_lib = None


def lib() -> C.CDLL:
    """Loads libtbik.so (built by ``python -m paper_2511_17826_amd.build``); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libtbik.so is not built: run `python -m paper_2511_17826_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


class TbikError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().tbik_status_string(status).decode()
        if status == 8:
            msg += " (hipError %d)" % lib().tbik_last_hip_error()
        super().__init__("%s: %s" % (where, msg))


def _check(status: int, where: str):
    if status != OK:
        raise TbikError(status, where)


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream() -> int:
    """Handle of torch's current stream on the current device (the raw getter saves about a microsecond per call)."""
    if _raw_stream is not None:
        return _raw_stream(torch.cuda.current_device())
    return torch.cuda.current_stream().cuda_stream


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return TBIK_F32
    if t.dtype == torch.bfloat16:
        return TBIK_BF16
    if t.dtype == torch.float16:
        return TBIK_F16
    raise TypeError("only float32, bfloat16 and float16 tensors are supported, got %s" % t.dtype)


def _rowmajor(t: torch.Tensor, name: str):
    if t.dim() != 2 or t.stride(1) != 1 or not t.is_cuda:
        raise ValueError("%s must be a 2-D row-major GPU tensor" % name)


_ws_cache = {}


def _workspace(nbytes: int, device) -> torch.Tensor:
    """A caller-side scratch tensor (the library itself never allocates), one per device AND stream: calls that share a
    workspace must not overlap in time, which only calls on one stream guarantee.  A tensor that is replaced by a larger
    one stays alive until the kernels already queued on its stream are done (torch's allocator frees a block for reuse
    by the stream it was allocated on).  Callers that run one call's kernels on several streams pass their own."""
    key = (str(device), _stream())
    w = _ws_cache.get(key)
    if w is None or w.numel() < nbytes:
        w = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        _ws_cache[key] = w
    return w


def gemm_workspace_bytes(M, N, K, leaf, k_first=1) -> int:
    return int(lib().tbik_gemm_workspace_bytes(M, N, K, leaf, k_first))


def _gemm(entry: str, in_dtype, X, W, leaf, k_first, out_dtype, out, workspace):
    _rowmajor(X, "X"); _rowmajor(W, "W")
    assert X.dtype == in_dtype and W.dtype == in_dtype
    M, K = X.shape
    K2, N = W.shape
    assert K == K2
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=X.device)
    _rowmajor(out, "out")
    if workspace is None:
        need = gemm_workspace_bytes(M, N, K, leaf, k_first)
        if need:
            workspace = _workspace(need, X.device)
    st = getattr(lib(), entry)(X.data_ptr(), X.stride(0), W.data_ptr(), W.stride(0), out.data_ptr(), out.stride(0),
                               _dt(out), M, N, K, leaf, k_first,
                               workspace.data_ptr() if workspace is not None else None,
                               workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream())
    _check(st, entry)
    return out


def tbik_gemm(X: torch.Tensor, W: torch.Tensor, leaf: int, k_first: int = 1, out_dtype=torch.bfloat16,
              out: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Y = X @ W in the tree order, whole K on this device (bf16 operands)."""
    return _gemm("tbik_gemm", torch.bfloat16, X, W, leaf, k_first, out_dtype, out, workspace)


def tbik_gemm_f16(X: torch.Tensor, W: torch.Tensor, leaf: int, k_first: int = 1, out_dtype=torch.float16,
                  out: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Y = X @ W in the tree order, whole K on this device (fp16 operands; fp16 or fp32 output)."""
    return _gemm("tbik_gemm_f16", torch.float16, X, W, leaf, k_first, out_dtype, out, workspace)


def tbik_gemm_f32(X: torch.Tensor, W: torch.Tensor, leaf: int, k_first: int = 1, out: torch.Tensor | None = None,
                  workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Y = X @ W in the tree order, whole K on this device (fp32 operands, fp32 output)."""
    _rowmajor(X, "X"); _rowmajor(W, "W")
    assert X.dtype == torch.float32 and W.dtype == torch.float32
    M, K = X.shape
    K2, N = W.shape
    assert K == K2
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=X.device)
    _rowmajor(out, "out")
    assert out.dtype == torch.float32 and out.shape == (M, N)
    if workspace is None:
        need = gemm_workspace_bytes(M, N, K, leaf, k_first)
        if need:
            workspace = _workspace(need, X.device)
    st = lib().tbik_gemm_f32(X.data_ptr(), X.stride(0), W.data_ptr(), W.stride(0), out.data_ptr(), out.stride(0),
                             M, N, K, leaf, k_first, workspace.data_ptr() if workspace is not None else None,
                             workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream())
    _check(st, "tbik_gemm_f32")
    return out


def _gemm_shard_partials(entry: str, in_dtype, X, W, leaf, k_first, P, out, workspace):
    _rowmajor(X, "X"); _rowmajor(W, "W")
    assert X.dtype == in_dtype and W.dtype == in_dtype
    M, K = X.shape
    N = W.shape[1]
    assert W.shape[0] == K
    if out is None:
        out = torch.empty((max(P, 1), M, N), dtype=torch.float32, device=X.device)
    assert out.is_contiguous() and out.dtype == torch.float32
    need = gemm_workspace_bytes(M, N, K, leaf, k_first)
    if workspace is None and need:
        workspace = _workspace(need, X.device)
    st = getattr(lib(), entry)(X.data_ptr(), X.stride(0), W.data_ptr(), W.stride(0), out.data_ptr(),
                               M, N, K, leaf, k_first, P,
                               workspace.data_ptr() if workspace is not None else None,
                               workspace.numel() * workspace.element_size() if workspace is not None else 0,
                               _stream())
    _check(st, entry)
    return out


def tbik_gemm_shard_partials(X: torch.Tensor, W: torch.Tensor, leaf: int, k_first: int, P: int,
                             out: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """partials[p] = subtree sum of K-shard p (fp32 [P, M, N]); bf16 operands."""
    return _gemm_shard_partials("tbik_gemm_shard_partials", torch.bfloat16, X, W, leaf, k_first, P, out, workspace)


def tbik_gemm_shard_partials_f16(X: torch.Tensor, W: torch.Tensor, leaf: int, k_first: int, P: int,
                                 out: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """partials[p] = subtree sum of K-shard p (fp32 [P, M, N]); fp16 operands."""
    return _gemm_shard_partials("tbik_gemm_shard_partials_f16", torch.float16, X, W, leaf, k_first, P, out, workspace)


def tbik_gemm_shard_partials_f32(X: torch.Tensor, W: torch.Tensor, leaf: int, k_first: int, P: int,
                                 out: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """partials[p] = subtree sum of K-shard p (fp32 [P, M, N]); fp32 operands."""
    return _gemm_shard_partials("tbik_gemm_shard_partials_f32", torch.float32, X, W, leaf, k_first, P, out, workspace)


TBIK_FP8_E4M3, TBIK_FP8_E5M2 = 3, 4
_FP8 = {"e4m3": TBIK_FP8_E4M3, "e5m2": TBIK_FP8_E5M2}


def _fp8_operands(X, Wt, fmt):
    """8-bit operands travel as uint8 tensors of patterns (or torch's float8 tensors, reinterpreted)."""
    def as_u8(t):
        return t if t.dtype == torch.uint8 else t.view(torch.uint8)
    X, Wt = as_u8(X), as_u8(Wt)
    _rowmajor(X, "X"); _rowmajor(Wt, "Wt")
    assert X.shape[1] == Wt.shape[1], "Wt is the transposed weight, [N, K]"
    return X, Wt, _FP8[fmt]


def gemm_fp8_workspace_bytes(M, N, K, leaf, k_first=1) -> int:
    return int(lib().tbik_gemm_fp8_workspace_bytes(M, N, K, leaf, k_first))


def tbik_gemm_fp8(X: torch.Tensor, Wt: torch.Tensor, leaf: int, k_first: int = 1, fmt: str = "e4m3",
                  out_dtype=torch.bfloat16, out: torch.Tensor | None = None, workspace: torch.Tensor | None = None):
    """Y = X @ Wt.T in the tree order on 8-bit floating-point operands; Wt is [N, K] (one row per output channel)."""
    X, Wt, dt = _fp8_operands(X, Wt, fmt)
    M, K = X.shape
    N = Wt.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=X.device)
    _rowmajor(out, "out")
    assert out.shape == (M, N)
    if workspace is None:
        need = gemm_fp8_workspace_bytes(M, N, K, leaf, k_first)
        if need:
            workspace = _workspace(need, X.device)
    st = lib().tbik_gemm_fp8(X.data_ptr(), X.stride(0), Wt.data_ptr(), Wt.stride(0), out.data_ptr(), out.stride(0),
                             _dt(out), dt, M, N, K, leaf, k_first, workspace.data_ptr() if workspace is not None else None,
                             workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream())
    _check(st, "tbik_gemm_fp8")
    return out


def tbik_gemm_shard_partials_fp8(X: torch.Tensor, Wt: torch.Tensor, leaf: int, k_first: int, P: int, fmt: str = "e4m3",
                                 out: torch.Tensor | None = None) -> torch.Tensor:
    X, Wt, dt = _fp8_operands(X, Wt, fmt)
    M, K = X.shape
    N = Wt.shape[0]
    if out is None:
        out = torch.empty((max(P, 1), M, N), dtype=torch.float32, device=X.device)
    assert out.is_contiguous() and out.dtype == torch.float32
    st = lib().tbik_gemm_shard_partials_fp8(X.data_ptr(), X.stride(0), Wt.data_ptr(), Wt.stride(0), out.data_ptr(), dt,
                                            M, N, K, leaf, k_first, P, None, 0, _stream())
    _check(st, "tbik_gemm_shard_partials_fp8")
    return out


def tbik_gemm_reference_fp8(X: torch.Tensor, Wt: torch.Tensor, leaf: int, k_first: int = 1, P: int = 1, fmt: str = "e4m3",
                            out_dtype=torch.float32):
    """The reference kernel: (Y, partials) for P == 1, partials alone otherwise."""
    X, Wt, dt = _fp8_operands(X, Wt, fmt)
    M, K = X.shape
    N = Wt.shape[0]
    parts = torch.empty((P, M, N), dtype=torch.float32, device=X.device)
    Y = torch.empty((M, N), dtype=out_dtype, device=X.device) if P == 1 else None
    st = lib().tbik_gemm_reference_fp8(X.data_ptr(), X.stride(0), Wt.data_ptr(), Wt.stride(0), parts.data_ptr(),
                                       Y.data_ptr() if Y is not None else None, N, _dt(Y) if Y is not None else TBIK_F32, dt,
                                       M, N, K, leaf, k_first, P, _stream())
    _check(st, "tbik_gemm_reference_fp8")
    return (Y, parts) if P == 1 else parts


def _mx_operands(X, Xs, Wt, Ws):
    for t, name in ((X, "X"), (Xs, "Xs"), (Wt, "Wt"), (Ws, "Ws")):
        _rowmajor(t, name)
        assert t.dtype == torch.uint8, "MXFP4 operands travel as uint8 tensors: packed element pairs and scale bytes"
    M, K2 = X.shape
    N = Wt.shape[0]
    K = 2 * K2
    assert Wt.shape[1] == K2 and Xs.shape == (M, K // 32) and Ws.shape == (N, K // 32)
    return M, N, K


def gemm_mxfp4_workspace_bytes(M, N, K, leaf, k_first=1) -> int:
    return int(lib().tbik_gemm_mxfp4_workspace_bytes(M, N, K, leaf, k_first))


def tbik_gemm_mxfp4(X, Xs, Wt, Ws, leaf: int, k_first: int = 1, out_dtype=torch.bfloat16, out: torch.Tensor | None = None,
                    workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Y = X @ Wt.T in the tree order on MXFP4 operands: X [M, K/2] packed pairs with scales Xs [M, K/32]; the weight
    transposed, Wt [N, K/2] with Ws [N, K/32]."""
    M, N, K = _mx_operands(X, Xs, Wt, Ws)
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=X.device)
    _rowmajor(out, "out")
    assert out.shape == (M, N)
    if workspace is None:
        need = gemm_mxfp4_workspace_bytes(M, N, K, leaf, k_first)
        if need:
            workspace = _workspace(need, X.device)
    st = lib().tbik_gemm_mxfp4(X.data_ptr(), X.stride(0), Xs.data_ptr(), Xs.stride(0), Wt.data_ptr(), Wt.stride(0),
                               Ws.data_ptr(), Ws.stride(0), out.data_ptr(), out.stride(0), _dt(out), M, N, K, leaf, k_first,
                               workspace.data_ptr() if workspace is not None else None,
                               workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream())
    _check(st, "tbik_gemm_mxfp4")
    return out


def tbik_gemm_shard_partials_mxfp4(X, Xs, Wt, Ws, leaf: int, k_first: int, P: int, out: torch.Tensor | None = None):
    M, N, K = _mx_operands(X, Xs, Wt, Ws)
    if out is None:
        out = torch.empty((max(P, 1), M, N), dtype=torch.float32, device=X.device)
    assert out.is_contiguous() and out.dtype == torch.float32
    need = gemm_mxfp4_workspace_bytes(M, N, K, leaf, k_first)
    ws = _workspace(need, X.device) if need else None
    st = lib().tbik_gemm_shard_partials_mxfp4(X.data_ptr(), X.stride(0), Xs.data_ptr(), Xs.stride(0), Wt.data_ptr(), Wt.stride(0),
                                              Ws.data_ptr(), Ws.stride(0), out.data_ptr(), M, N, K, leaf, k_first, P,
                                              ws.data_ptr() if ws is not None else None, need, _stream())
    _check(st, "tbik_gemm_shard_partials_mxfp4")
    return out


def tbik_gemm_reference_mxfp4(X, Xs, Wt, Ws, leaf: int, k_first: int = 1, P: int = 1, out_dtype=torch.float32):
    """The reference kernel: (Y, partials) for P == 1, partials alone otherwise."""
    M, N, K = _mx_operands(X, Xs, Wt, Ws)
    parts = torch.empty((P, M, N), dtype=torch.float32, device=X.device)
    Y = torch.empty((M, N), dtype=out_dtype, device=X.device) if P == 1 else None
    st = lib().tbik_gemm_reference_mxfp4(X.data_ptr(), X.stride(0), Xs.data_ptr(), Xs.stride(0), Wt.data_ptr(), Wt.stride(0),
                                         Ws.data_ptr(), Ws.stride(0), parts.data_ptr(), Y.data_ptr() if Y is not None else None, N,
                                         _dt(Y) if Y is not None else TBIK_F32, M, N, K, leaf, k_first, P, _stream())
    _check(st, "tbik_gemm_reference_mxfp4")
    return (Y, parts) if P == 1 else parts


def _mx8_operands(X, Xs, Wt, Ws, fmt):
    X, Wt, dt = _fp8_operands(X, Wt, fmt)
    for t, name in ((Xs, "Xs"), (Ws, "Ws")):
        _rowmajor(t, name)
        assert t.dtype == torch.uint8, "E8M0 scales travel as uint8 tensors"
    M, K = X.shape
    N = Wt.shape[0]
    assert Xs.shape == (M, K // 32) and Ws.shape == (N, K // 32)
    return X, Wt, dt, M, N, K


def gemm_mxfp8_workspace_bytes(M, N, K, leaf, k_first=1) -> int:
    return int(lib().tbik_gemm_mxfp8_workspace_bytes(M, N, K, leaf, k_first))


def tbik_gemm_mxfp8(X, Xs, Wt, Ws, leaf: int, k_first: int = 1, fmt: str = "e4m3", out_dtype=torch.bfloat16,
                    out: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Y = X @ Wt.T in the tree order on MXFP8 operands: X [M, K] 8-bit patterns of format `fmt` with scales Xs [M, K/32];
    the weight transposed, Wt [N, K] with Ws [N, K/32]."""
    X, Wt, dt, M, N, K = _mx8_operands(X, Xs, Wt, Ws, fmt)
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=X.device)
    _rowmajor(out, "out")
    assert out.shape == (M, N)
    if workspace is None:
        need = gemm_mxfp8_workspace_bytes(M, N, K, leaf, k_first)
        if need:
            workspace = _workspace(need, X.device)
    st = lib().tbik_gemm_mxfp8(X.data_ptr(), X.stride(0), Xs.data_ptr(), Xs.stride(0), Wt.data_ptr(), Wt.stride(0),
                               Ws.data_ptr(), Ws.stride(0), out.data_ptr(), out.stride(0), _dt(out), dt, M, N, K, leaf, k_first,
                               workspace.data_ptr() if workspace is not None else None,
                               workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream())
    _check(st, "tbik_gemm_mxfp8")
    return out


def tbik_gemm_shard_partials_mxfp8(X, Xs, Wt, Ws, leaf: int, k_first: int, P: int, fmt: str = "e4m3",
                                   out: torch.Tensor | None = None):
    X, Wt, dt, M, N, K = _mx8_operands(X, Xs, Wt, Ws, fmt)
    if out is None:
        out = torch.empty((max(P, 1), M, N), dtype=torch.float32, device=X.device)
    assert out.is_contiguous() and out.dtype == torch.float32
    need = gemm_mxfp8_workspace_bytes(M, N, K, leaf, k_first)
    ws = _workspace(need, X.device) if need else None
    st = lib().tbik_gemm_shard_partials_mxfp8(X.data_ptr(), X.stride(0), Xs.data_ptr(), Xs.stride(0), Wt.data_ptr(), Wt.stride(0),
                                              Ws.data_ptr(), Ws.stride(0), out.data_ptr(), dt, M, N, K, leaf, k_first, P,
                                              ws.data_ptr() if ws is not None else None, need, _stream())
    _check(st, "tbik_gemm_shard_partials_mxfp8")
    return out


def tbik_gemm_reference_mxfp8(X, Xs, Wt, Ws, leaf: int, k_first: int = 1, P: int = 1, fmt: str = "e4m3",
                              out_dtype=torch.float32):
    """The reference kernel: (Y, partials) for P == 1, partials alone otherwise."""
    X, Wt, dt, M, N, K = _mx8_operands(X, Xs, Wt, Ws, fmt)
    parts = torch.empty((P, M, N), dtype=torch.float32, device=X.device)
    Y = torch.empty((M, N), dtype=out_dtype, device=X.device) if P == 1 else None
    st = lib().tbik_gemm_reference_mxfp8(X.data_ptr(), X.stride(0), Xs.data_ptr(), Xs.stride(0), Wt.data_ptr(), Wt.stride(0),
                                         Ws.data_ptr(), Ws.stride(0), parts.data_ptr(), Y.data_ptr() if Y is not None else None, N,
                                         _dt(Y) if Y is not None else TBIK_F32, dt, M, N, K, leaf, k_first, P, _stream())
    _check(st, "tbik_gemm_reference_mxfp8")
    return (Y, parts) if P == 1 else parts


TBIK_FP6_E2M3, TBIK_FP6_E3M2 = 6, 7
_FP6 = {"e2m3": TBIK_FP6_E2M3, "e3m2": TBIK_FP6_E3M2}


def _mx6_operands(X, Xs, Wt, Ws, fmt):
    for t, name in ((X, "X"), (Xs, "Xs"), (Wt, "Wt"), (Ws, "Ws")):
        _rowmajor(t, name)
        assert t.dtype == torch.uint8, "MXFP6 operands travel as uint8 tensors: packed 6-bit elements and scale bytes"
    M, KB = X.shape
    N = Wt.shape[0]
    K = KB * 4 // 3
    assert KB * 4 == K * 3 and Wt.shape[1] == KB and Xs.shape == (M, K // 32) and Ws.shape == (N, K // 32)
    return _FP6[fmt], M, N, K


def gemm_mxfp6_workspace_bytes(M, N, K, leaf, k_first=1) -> int:
    return int(lib().tbik_gemm_mxfp6_workspace_bytes(M, N, K, leaf, k_first))


def tbik_gemm_mxfp6(X, Xs, Wt, Ws, leaf: int, k_first: int = 1, fmt: str = "e2m3", out_dtype=torch.bfloat16,
                    out: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Y = X @ Wt.T in the tree order on MXFP6 operands: X [M, 3K/4] packed 6-bit elements of format `fmt` with scales
    Xs [M, K/32]; the weight transposed, Wt [N, 3K/4] with Ws [N, K/32]."""
    dt, M, N, K = _mx6_operands(X, Xs, Wt, Ws, fmt)
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=X.device)
    _rowmajor(out, "out")
    assert out.shape == (M, N)
    if workspace is None:
        need = gemm_mxfp6_workspace_bytes(M, N, K, leaf, k_first)
        if need:
            workspace = _workspace(need, X.device)
    st = lib().tbik_gemm_mxfp6(X.data_ptr(), X.stride(0), Xs.data_ptr(), Xs.stride(0), Wt.data_ptr(), Wt.stride(0),
                               Ws.data_ptr(), Ws.stride(0), out.data_ptr(), out.stride(0), _dt(out), dt, M, N, K, leaf, k_first,
                               workspace.data_ptr() if workspace is not None else None,
                               workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream())
    _check(st, "tbik_gemm_mxfp6")
    return out


def tbik_gemm_shard_partials_mxfp6(X, Xs, Wt, Ws, leaf: int, k_first: int, P: int, fmt: str = "e2m3",
                                   out: torch.Tensor | None = None):
    dt, M, N, K = _mx6_operands(X, Xs, Wt, Ws, fmt)
    if out is None:
        out = torch.empty((max(P, 1), M, N), dtype=torch.float32, device=X.device)
    assert out.is_contiguous() and out.dtype == torch.float32
    need = gemm_mxfp6_workspace_bytes(M, N, K, leaf, k_first)
    ws = _workspace(need, X.device) if need else None
    st = lib().tbik_gemm_shard_partials_mxfp6(X.data_ptr(), X.stride(0), Xs.data_ptr(), Xs.stride(0), Wt.data_ptr(), Wt.stride(0),
                                              Ws.data_ptr(), Ws.stride(0), out.data_ptr(), dt, M, N, K, leaf, k_first, P,
                                              ws.data_ptr() if ws is not None else None, need, _stream())
    _check(st, "tbik_gemm_shard_partials_mxfp6")
    return out


def tbik_gemm_reference_mxfp6(X, Xs, Wt, Ws, leaf: int, k_first: int = 1, P: int = 1, fmt: str = "e2m3",
                              out_dtype=torch.float32):
    """The reference kernel: (Y, partials) for P == 1, partials alone otherwise."""
    dt, M, N, K = _mx6_operands(X, Xs, Wt, Ws, fmt)
    parts = torch.empty((P, M, N), dtype=torch.float32, device=X.device)
    Y = torch.empty((M, N), dtype=out_dtype, device=X.device) if P == 1 else None
    st = lib().tbik_gemm_reference_mxfp6(X.data_ptr(), X.stride(0), Xs.data_ptr(), Xs.stride(0), Wt.data_ptr(), Wt.stride(0),
                                         Ws.data_ptr(), Ws.stride(0), parts.data_ptr(), Y.data_ptr() if Y is not None else None, N,
                                         _dt(Y) if Y is not None else TBIK_F32, dt, M, N, K, leaf, k_first, P, _stream())
    _check(st, "tbik_gemm_reference_mxfp6")
    return (Y, parts) if P == 1 else parts


def tbik_tree_allreduce(bufs: torch.Tensor) -> torch.Tensor:
    """Alg. 2 round by round, in place, on rank buffers [P, ...] (fp32, contiguous): every buffer ends up holding T."""
    assert bufs.is_cuda and bufs.is_contiguous() and bufs.dtype == torch.float32 and bufs.dim() >= 1
    P = bufs.shape[0]
    n = bufs.numel() // max(P, 1)
    _check(lib().tbik_tree_allreduce(bufs.data_ptr(), P, n, _stream()), "tbik_tree_allreduce")
    return bufs


def tbik_silu_mul(gate: torch.Tensor, up: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """act = SiLU(gate) * up on [M, I] bf16 or fp16 tensors (row-major; views into one [M, 2 I] buffer are fine)."""
    _rowmajor(gate, "gate"); _rowmajor(up, "up")
    assert gate.dtype == up.dtype and gate.dtype in (torch.bfloat16, torch.float16) and gate.shape == up.shape
    M, I = gate.shape
    if out is None:
        out = torch.empty((M, I), dtype=gate.dtype, device=gate.device)
    _rowmajor(out, "out")
    assert out.dtype == gate.dtype and out.shape == (M, I)
    st = lib().tbik_silu_mul(gate.data_ptr(), gate.stride(0), up.data_ptr(), up.stride(0), out.data_ptr(), out.stride(0),
                             _dt(gate), M, I, _stream())
    _check(st, "tbik_silu_mul")
    return out


def gemm_swiglu_workspace_bytes(M, I, K, leaf, k_first=1) -> int:
    return int(lib().tbik_gemm_swiglu_workspace_bytes(M, I, K, leaf, k_first))


def tbik_gemm_swiglu(X: torch.Tensor, W_gu: torch.Tensor, leaf: int, k_first: int = 1, out: torch.Tensor | None = None,
                     workspace: torch.Tensor | None = None) -> torch.Tensor:
    """act = SiLU(X @ W_gu[:, :I]) * (X @ W_gu[:, I:]) in the tree order; W_gu is [K, 2 I], gate columns first."""
    _rowmajor(X, "X"); _rowmajor(W_gu, "W_gu")
    assert X.dtype == W_gu.dtype and X.dtype in (torch.bfloat16, torch.float16)
    M, K = X.shape
    assert W_gu.shape[0] == K and W_gu.shape[1] % 2 == 0
    I = W_gu.shape[1] // 2
    if out is None:
        out = torch.empty((M, I), dtype=X.dtype, device=X.device)
    _rowmajor(out, "out")
    assert out.dtype == X.dtype and out.shape == (M, I)
    if workspace is None:
        need = gemm_swiglu_workspace_bytes(M, I, K, leaf, k_first)
        if need:
            workspace = _workspace(need, X.device)
    st = lib().tbik_gemm_swiglu(X.data_ptr(), X.stride(0), W_gu.data_ptr(), W_gu.stride(0), out.data_ptr(), out.stride(0),
                                _dt(X), M, I, K, leaf, k_first, workspace.data_ptr() if workspace is not None else None,
                                workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream())
    _check(st, "tbik_gemm_swiglu")
    return out


def tbik_tree_combine(partials: torch.Tensor, out_dtype=torch.bfloat16, out: torch.Tensor | None = None) -> torch.Tensor:
    """Y = T(partials[0..P)) elementwise, one rounding to the output type."""
    assert partials.dim() == 3 and partials.is_contiguous() and partials.dtype == torch.float32
    P, M, N = partials.shape
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=partials.device)
    _rowmajor(out, "out")
    st = lib().tbik_tree_combine(partials.data_ptr(), P, out.data_ptr(), out.stride(0), _dt(out), M, N, _stream())
    _check(st, "tbik_tree_combine")
    return out


def _rmsnorm(name, dtype, x, weight, eps, out):
    assert x.dim() == 2 and x.is_contiguous() and x.dtype == dtype
    assert weight.is_contiguous() and weight.dtype == dtype and weight.numel() == x.shape[1]
    if out is None:
        out = torch.empty_like(x)
    assert out.shape == x.shape and out.is_contiguous() and out.dtype == dtype
    st = getattr(lib(), name)(x.data_ptr(), weight.data_ptr(), out.data_ptr(), x.shape[0], x.shape[1], eps, _stream())
    _check(st, name)
    return out


def tbik_rmsnorm(x: torch.Tensor, weight: torch.Tensor, eps: float = 1e-6, out: torch.Tensor | None = None) -> torch.Tensor:
    return _rmsnorm("tbik_rmsnorm", torch.bfloat16, x, weight, eps, out)


def tbik_rmsnorm_f16(x: torch.Tensor, weight: torch.Tensor, eps: float = 1e-6, out: torch.Tensor | None = None) -> torch.Tensor:
    return _rmsnorm("tbik_rmsnorm_f16", torch.float16, x, weight, eps, out)


def _combine_residual_rmsnorm(name, dtype, partials, residual, weight, eps, hidden, normed):
    assert partials.dim() == 3 and partials.is_contiguous() and partials.dtype == torch.float32
    P, M, H = partials.shape
    assert residual.shape == (M, H) and residual.is_contiguous() and residual.dtype == dtype
    assert weight.shape == (H,) and weight.dtype == dtype
    if hidden is None:
        hidden = torch.empty_like(residual)
    if normed is None:
        normed = torch.empty_like(residual)
    assert hidden.is_contiguous() and normed.is_contiguous() and hidden.dtype == normed.dtype == dtype
    assert hidden.shape == normed.shape == (M, H)
    st = getattr(lib(), name)(partials.data_ptr(), P, residual.data_ptr(), weight.data_ptr(), eps,
                              hidden.data_ptr(), normed.data_ptr(), M, H, _stream())
    _check(st, name)
    return hidden, normed


def tbik_combine_residual_rmsnorm(partials: torch.Tensor, residual: torch.Tensor, weight: torch.Tensor, eps: float = 1e-6,
                                  hidden: torch.Tensor | None = None, normed: torch.Tensor | None = None):
    """(hidden, normed): hidden = bf16(bf16(T(partials)) + residual), normed = RMSNorm(hidden); one kernel."""
    return _combine_residual_rmsnorm("tbik_combine_residual_rmsnorm", torch.bfloat16, partials, residual, weight, eps,
                                     hidden, normed)


def tbik_combine_residual_rmsnorm_f16(partials: torch.Tensor, residual: torch.Tensor, weight: torch.Tensor,
                                      eps: float = 1e-6, hidden: torch.Tensor | None = None,
                                      normed: torch.Tensor | None = None):
    """The same with fp16 residual, weight and outputs."""
    return _combine_residual_rmsnorm("tbik_combine_residual_rmsnorm_f16", torch.float16, partials, residual, weight, eps,
                                     hidden, normed)


def _token_major(t: torch.Tensor, name: str, dtype):
    if t.dim() != 3 or t.stride(2) != 1 or t.stride(1) != t.shape[2] or not t.is_cuda or t.dtype != dtype:
        raise ValueError("%s must be a %s GPU tensor [tokens, heads, head_dim] with contiguous heads" % (name, dtype))


def attention_workspace_bytes(batch, max_seqlen_q, max_seqlen_k, heads_q, heads_kv) -> int:
    return int(lib().tbik_attention_workspace_bytes(batch, max_seqlen_q, max_seqlen_k, heads_q, heads_kv))


def _attention(entry, dtype, Q, K, V, cu_seqlens_q, cu_seqlens_k, max_seqlen_q, scale, causal, out, max_seqlen_k, workspace,
               verify_lengths=False):
    _token_major(Q, "Q", dtype); _token_major(K, "K", dtype); _token_major(V, "V", dtype)
    Tq, Hq, D = Q.shape
    Tk, Hkv, _ = K.shape
    assert V.shape == K.shape and K.shape[2] == D
    assert cu_seqlens_q.dtype == torch.int32 and cu_seqlens_k.dtype == torch.int32
    assert cu_seqlens_q.is_cuda and cu_seqlens_k.is_cuda and cu_seqlens_q.is_contiguous() and cu_seqlens_k.is_contiguous()
    assert cu_seqlens_q.numel() == cu_seqlens_k.numel() >= 1
    if out is None:
        out = torch.empty((Tq, Hq, D), dtype=dtype, device=Q.device)
    _token_major(out, "out", dtype)
    assert out.shape == Q.shape
    batch = cu_seqlens_q.numel() - 1
    if max_seqlen_k is None:                          # not given: read it from the device (a synchronisation)
        max_seqlen_k = int((cu_seqlens_k[1:] - cu_seqlens_k[:-1]).max().item()) if batch > 0 else 0
    elif verify_lengths and batch > 0:                # an understated bound leaves keys out without an error: check it here
        longest = int((cu_seqlens_k[1:] - cu_seqlens_k[:-1]).max().item())
        if longest > max_seqlen_k:
            raise ValueError("max_seqlen_k = %d, but a sequence has %d keys" % (max_seqlen_k, longest))
    need = int(lib().tbik_attention_workspace_bytes(batch, max_seqlen_q, min(max_seqlen_k, Tk), Hq, Hkv)) if D == 128 else 0
    if workspace is None and need:
        workspace = _workspace(need, Q.device)
    st = getattr(lib(), entry)(Q.data_ptr(), K.data_ptr(), V.data_ptr(), out.data_ptr(), cu_seqlens_q.data_ptr(),
                               cu_seqlens_k.data_ptr(), batch, max_seqlen_q, max_seqlen_k, Tq, Tk, Hq, Hkv, D,
                               Q.stride(0), K.stride(0), V.stride(0), out.stride(0), scale, int(causal),
                               workspace.data_ptr() if workspace is not None else None,
                               workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream())
    _check(st, entry)
    return out


def tbik_attention(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, cu_seqlens_q: torch.Tensor,
                   cu_seqlens_k: torch.Tensor, max_seqlen_q: int, scale: float, causal: bool = True,
                   out: torch.Tensor | None = None, max_seqlen_k: int | None = None,
                   workspace: torch.Tensor | None = None, verify_lengths: bool = False) -> torch.Tensor:
    """Fixed-tile, fixed-split attention on packed sequences: Q [Tq, Hq, D], K and V [Tk, Hkv, D] (token stride free),
    cu_seqlens_* int32 GPU tensors [batch + 1].  Returns O [Tq, Hq, D] bf16.  `max_seqlen_k` must be at least the longest
    sequence's key count (the C call cannot see the lengths, which live on the device: keys past an understated bound
    are left out of the softmax without an error); `verify_lengths` checks it against `cu_seqlens_k` at the cost of a
    synchronisation, and leaving `max_seqlen_k` out reads it from there."""
    return _attention("tbik_attention", torch.bfloat16, Q, K, V, cu_seqlens_q, cu_seqlens_k, max_seqlen_q, scale, causal, out,
                      max_seqlen_k, workspace, verify_lengths)


def tbik_attention_f16(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, cu_seqlens_q: torch.Tensor,
                       cu_seqlens_k: torch.Tensor, max_seqlen_q: int, scale: float, causal: bool = True,
                       out: torch.Tensor | None = None, max_seqlen_k: int | None = None,
                       workspace: torch.Tensor | None = None, verify_lengths: bool = False) -> torch.Tensor:
    """The same on fp16 tensors."""
    return _attention("tbik_attention_f16", torch.float16, Q, K, V, cu_seqlens_q, cu_seqlens_k, max_seqlen_q, scale, causal, out,
                      max_seqlen_k, workspace, verify_lengths)


def tbik_row_reduce(x: torch.Tensor, op: int, out: torch.Tensor | None = None,
                    workspace: torch.Tensor | None = None) -> torch.Tensor:
    """op = TBIK_SUM / TBIK_MAX -> fp32 [M]; TBIK_LOGSOFTMAX -> fp32 [M, V]."""
    assert x.dim() == 2 and x.is_contiguous()
    M, V = x.shape
    if out is None:
        out = torch.empty((M, V) if op == TBIK_LOGSOFTMAX else (M,), dtype=torch.float32, device=x.device)
    need = int(lib().tbik_row_reduce_workspace_bytes(M, V, op))
    if workspace is None:
        workspace = _workspace(need, x.device)
    st = lib().tbik_row_reduce(x.data_ptr(), _dt(x), out.data_ptr(), op, M, V, workspace.data_ptr(),
                               workspace.numel() * workspace.element_size(), _stream())
    _check(st, "tbik_row_reduce")
    return out


def tbik_row_reduce_static(x: torch.Tensor, op: int, out: torch.Tensor) -> torch.Tensor:
    """tbik_row_reduce on the library's fixed scratch array: no workspace, no allocation (``out`` is the caller's)."""
    assert x.dim() == 2 and x.is_contiguous() and out.is_contiguous() and out.dtype == torch.float32
    M, V = x.shape
    assert out.numel() == (M * V if op == TBIK_LOGSOFTMAX else M)
    st = lib().tbik_row_reduce_static(x.data_ptr(), _dt(x), out.data_ptr(), op, M, V, _stream())
    _check(st, "tbik_row_reduce_static")
    return out


def tbik_gemm_reference(X: torch.Tensor, W: torch.Tensor, leaf: int, k_first: int = 1, P: int = 1,
                        out_dtype=torch.float32):
    """The reference kernel: returns (partials [P,M,N] fp32, Y or None); Y only for P == 1."""
    return _gemm_reference("tbik_gemm_reference", torch.bfloat16, X, W, leaf, k_first, P, out_dtype)


def tbik_gemm_reference_f16(X: torch.Tensor, W: torch.Tensor, leaf: int, k_first: int = 1, P: int = 1,
                            out_dtype=torch.float32):
    """The reference kernel on fp16 operands."""
    return _gemm_reference("tbik_gemm_reference_f16", torch.float16, X, W, leaf, k_first, P, out_dtype)


def tbik_gemm_reference_f32(X: torch.Tensor, W: torch.Tensor, leaf: int, k_first: int = 1, P: int = 1):
    """The reference kernel on fp32 operands: (partials [P,M,N], Y fp32 or None)."""
    _rowmajor(X, "X"); _rowmajor(W, "W")
    assert X.dtype == torch.float32 and W.dtype == torch.float32
    M, K = X.shape
    N = W.shape[1]
    parts = torch.empty((P, M, N), dtype=torch.float32, device=X.device)
    Y = torch.empty((M, N), dtype=torch.float32, device=X.device) if P == 1 else None
    st = lib().tbik_gemm_reference_f32(X.data_ptr(), X.stride(0), W.data_ptr(), W.stride(0), parts.data_ptr(),
                                       Y.data_ptr() if Y is not None else None, Y.stride(0) if Y is not None else 0,
                                       M, N, K, leaf, k_first, P, _stream())
    _check(st, "tbik_gemm_reference_f32")
    return parts, Y


def _gemm_reference(entry: str, in_dtype, X, W, leaf, k_first, P, out_dtype):
    _rowmajor(X, "X"); _rowmajor(W, "W")
    assert X.dtype == in_dtype and W.dtype == in_dtype
    M, K = X.shape
    N = W.shape[1]
    parts = torch.empty((P, M, N), dtype=torch.float32, device=X.device)
    Y = torch.empty((M, N), dtype=out_dtype, device=X.device) if P == 1 else None
    st = getattr(lib(), entry)(X.data_ptr(), X.stride(0), W.data_ptr(), W.stride(0), parts.data_ptr(),
                               Y.data_ptr() if Y is not None else None, Y.stride(0) if Y is not None else 0,
                               _dt(Y) if Y is not None else TBIK_F32, M, N, K, leaf, k_first, P, _stream())
    _check(st, entry)
    return parts, Y


def tbik_set_row_wait_limit(polls: int) -> int:
    """Bound of the inter-workgroup waits of the long-row log-softmax (testing); returns the previous bound."""
    return int(lib().tbik_set_row_wait_limit(polls))


def tbik_set_attention_variant(variant: int):
    _check(lib().tbik_set_attention_variant(variant), "tbik_set_attention_variant")


def tbik_set_gemm_variant(variant: int):
    _check(lib().tbik_set_gemm_variant(variant), "tbik_set_gemm_variant")


def variant_names():
    out, i = [], 0
    while True:
        n = lib().tbik_variant_name(i)
        if n is None:
            return out
        out.append(n.decode())
        i += 1
