"""ctypes binding of libflashbias.so: argument marshalling only.

Function names and argument order mirror include/flashbias.h.  Tensors are torch CUDA
tensors used purely as device buffers (data_ptr, dtype, shape); every step of the
computation runs inside the library's HIP kernels.  There is no fallback: if the shared
library is missing or a call returns an error status, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflashbias.so")

FB_F32, FB_BF16 = 0, 1
_lib_handle = None

EXPORTS = (
    "fb_version", "fb_status_string", "fb_tune_set", "fb_lowrank_attn_fwd", "fb_lowrank_xattn_fwd",
    "fb_alibi_attn_fwd", "fb_dense_bias_attn_fwd", "fb_lowrank_attn_bwd_workspace_bytes",
    "fb_lowrank_attn_bwd", "fb_lowrank_xattn_bwd_workspace_bytes", "fb_lowrank_xattn_bwd",
    "fb_dense_bias_attn_bwd_workspace_bytes", "fb_dense_bias_attn_bwd",
    "fb_lowrank_mulbias_attn_fwd_workspace_bytes", "fb_lowrank_mulbias_attn_fwd",
    "fb_lowrank_mulbias_attn_bwd_workspace_bytes", "fb_lowrank_mulbias_attn_bwd",
    "fb_alibi_attn_bwd_workspace_bytes", "fb_alibi_attn_bwd", "fb_lowrank_attn_bwd_noalloc",
)

FB_STATIC_SCRATCH_BYTES = 64 << 20     # include/flashbias.h


class FlashBiasError(RuntimeError):
    pass


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load (once) and type the C-ABI.  Raises FlashBiasError if the library is not built."""
    global _lib_handle
    if _lib_handle is not None and path is None:
        return _lib_handle
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise FlashBiasError(
            f"{p} not found: build it first (python -m paper_2505_12044_amd.build or "
            "__graft_entry__.build()); there is no CPU fallback")
    lib = ctypes.CDLL(p)
    vp, ci, cf, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.fb_version.restype = ci
    lib.fb_version.argtypes = []
    lib.fb_status_string.restype = ctypes.c_char_p
    lib.fb_status_string.argtypes = [ci]
    lib.fb_tune_set.restype = ci
    lib.fb_tune_set.argtypes = [ctypes.c_char_p, ci]
    lib.fb_lowrank_attn_fwd.restype = ci
    lib.fb_lowrank_attn_fwd.argtypes = [vp] * 7 + [ci] * 6 + [ci, ci, ci, cf, vp]
    lib.fb_lowrank_xattn_fwd.restype = ci
    lib.fb_lowrank_xattn_fwd.argtypes = [vp] * 7 + [ci] * 6 + [ci, ci, ci, cf, vp]
    lib.fb_alibi_attn_fwd.restype = ci
    lib.fb_alibi_attn_fwd.argtypes = [vp] * 6 + [ci] * 5 + [ci, cf, vp]
    lib.fb_dense_bias_attn_fwd.restype = ci
    lib.fb_dense_bias_attn_fwd.argtypes = [vp] * 6 + [ci] * 5 + [ci, ci, cf, vp]
    lib.fb_lowrank_attn_bwd_workspace_bytes.restype = sz
    lib.fb_lowrank_attn_bwd_workspace_bytes.argtypes = [ci] * 5 + [ci]
    lib.fb_lowrank_attn_bwd.restype = ci
    lib.fb_lowrank_attn_bwd.argtypes = [vp] * 13 + [ci] * 6 + [ci, ci, ci, cf, vp, sz, vp]
    lib.fb_lowrank_attn_bwd_noalloc.restype = ci
    lib.fb_lowrank_attn_bwd_noalloc.argtypes = [vp] * 13 + [ci] * 6 + [ci, ci, ci, cf, vp]
    lib.fb_dense_bias_attn_bwd_workspace_bytes.restype = sz
    lib.fb_dense_bias_attn_bwd_workspace_bytes.argtypes = [ci] * 4 + [ci]
    lib.fb_dense_bias_attn_bwd.restype = ci
    lib.fb_dense_bias_attn_bwd.argtypes = [vp] * 11 + [ci] * 5 + [ci, ci, cf, vp, sz, vp]
    lib.fb_lowrank_xattn_bwd_workspace_bytes.restype = sz
    lib.fb_lowrank_xattn_bwd_workspace_bytes.argtypes = [ci] * 6 + [ci]
    lib.fb_lowrank_xattn_bwd.restype = ci
    lib.fb_lowrank_xattn_bwd.argtypes = [vp] * 13 + [ci] * 6 + [ci, ci, ci, cf, vp, sz, vp]
    lib.fb_lowrank_mulbias_attn_fwd_workspace_bytes.restype = sz
    lib.fb_lowrank_mulbias_attn_fwd_workspace_bytes.argtypes = [ci] * 5 + [ci]
    lib.fb_lowrank_mulbias_attn_fwd.restype = ci
    lib.fb_lowrank_mulbias_attn_fwd.argtypes = [vp] * 7 + [ci] * 6 + [ci, ci, ci, cf, vp, sz, vp]
    lib.fb_lowrank_mulbias_attn_bwd_workspace_bytes.restype = sz
    lib.fb_lowrank_mulbias_attn_bwd_workspace_bytes.argtypes = [ci] * 5 + [ci]
    lib.fb_lowrank_mulbias_attn_bwd.restype = ci
    lib.fb_lowrank_mulbias_attn_bwd.argtypes = [vp] * 13 + [ci] * 6 + [ci, ci, ci, cf, vp, sz, vp]
    lib.fb_alibi_attn_bwd_workspace_bytes.restype = sz
    lib.fb_alibi_attn_bwd_workspace_bytes.argtypes = [ci] * 4 + [ci]
    lib.fb_alibi_attn_bwd.restype = ci
    lib.fb_alibi_attn_bwd.argtypes = [vp] * 11 + [ci] * 5 + [ci, cf, vp, sz, vp]
    if path is None:
        _lib_handle = lib
    return lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return FB_F32
    if t.dtype == torch.bfloat16:
        return FB_BF16
    raise FlashBiasError(f"unsupported tensor dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise FlashBiasError("tensors must be contiguous CUDA tensors")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    h = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
    return h or None


def _scratch(nbytes: int, device, stream) -> torch.Tensor:
    """A workspace the wrapper allocates itself.  The kernels run on `stream`; when that is not
    torch's current stream the caching allocator must be told, or it could hand the block to
    other work as soon as the tensor is dropped."""
    ws = torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)
    if stream is not None and hasattr(stream, "cuda_stream") and stream != torch.cuda.current_stream():
        ws.record_stream(stream)
    return ws


def _check(status: int, what: str) -> None:
    if status != 0:
        msg = load_library().fb_status_string(status).decode()
        raise FlashBiasError(f"{what} failed: status {status} ({msg})")


def fb_version() -> int:
    return load_library().fb_version()


def fb_tune_set(name: str, value: int) -> None:
    _check(load_library().fb_tune_set(name.encode(), int(value)), "fb_tune_set")


def fb_lowrank_attn_fwd(q, k, v, phi_q, phi_k, out=None, lse=None, causal=False,
                        scale: float = 0.0, phi_batch_broadcast: Optional[bool] = None,
                        stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """out, lse = attention(q, k, v) with bias phi_q phi_k^T.  q, k, v: [B,H,N,C];
    phi_q, phi_k: [B or 1,H,N,R] (None for R = 0)."""
    lib = load_library()
    B, H, N, C = q.shape
    R = 0 if phi_q is None else phi_q.shape[-1]
    if phi_batch_broadcast is None:
        phi_batch_broadcast = phi_q is not None and phi_q.shape[0] == 1 and B > 1
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    phi_code = _dtype_code(phi_q) if phi_q is not None else _dtype_code(q)
    st = lib.fb_lowrank_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(phi_q), _ptr(phi_k), _ptr(out),
                                 _ptr(lse), B, H, N, C, R, int(bool(causal)), _dtype_code(q),
                                 phi_code, int(bool(phi_batch_broadcast)), float(scale),
                                 _stream(stream))
    _check(st, "fb_lowrank_attn_fwd")
    return out, lse


def fb_lowrank_xattn_fwd(q, k, v, phi_q, phi_k, out=None, lse=None, scale: float = 0.0,
                         phi_batch_broadcast: Optional[bool] = None, stream=None):
    """Cross-attention: q [B,H,N,C], k, v [B,H,M,C], phi_q [B or 1,H,N,R], phi_k [B or 1,H,M,R]."""
    lib = load_library()
    B, H, N, C = q.shape
    M = k.shape[2]
    R = 0 if phi_q is None else phi_q.shape[-1]
    if phi_batch_broadcast is None:
        phi_batch_broadcast = phi_q is not None and phi_q.shape[0] == 1 and B > 1
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    phi_code = _dtype_code(phi_q) if phi_q is not None else _dtype_code(q)
    st = lib.fb_lowrank_xattn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(phi_q), _ptr(phi_k), _ptr(out),
                                  _ptr(lse), B, H, N, M, C, R, _dtype_code(q), phi_code,
                                  int(bool(phi_batch_broadcast)), float(scale), _stream(stream))
    _check(st, "fb_lowrank_xattn_fwd")
    return out, lse


def fb_alibi_attn_bwd_workspace_bytes(B, H, N, C, dtype_code=FB_BF16) -> int:
    return int(load_library().fb_alibi_attn_bwd_workspace_bytes(B, H, N, C, dtype_code))


def fb_alibi_attn_bwd(q, k, v, slopes, out, lse, dout, causal=False, scale: float = 0.0, workspace=None,
                      grads=None, dslope_rows=None, stream=None):
    """dq, dk, dv of the attention with the in-kernel ALiBi bias -slopes[h] * (i - j).  dslope_rows: optional
    [B,H,N] float32 tensor that receives each query row's contribution to dL/dslope[h]."""
    lib = load_library()
    B, H, N, C = q.shape
    if slopes.dtype != torch.float32 or slopes.numel() != H:
        raise FlashBiasError("slopes must be a float32 tensor with one entry per head")
    need = fb_alibi_attn_bwd_workspace_bytes(B, H, N, C)
    if workspace is None:
        workspace = _scratch(need, q.device, stream)
    if grads is None:
        grads = (torch.empty_like(q), torch.empty_like(k), torch.empty_like(v))
    dq, dk, dv = grads
    st = lib.fb_alibi_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(slopes), _ptr(out), _ptr(lse), _ptr(dout),
                               _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dslope_rows), B, H, N, C, int(bool(causal)),
                               _dtype_code(q), float(scale), _ptr(workspace), workspace.numel(), _stream(stream))
    _check(st, "fb_alibi_attn_bwd")
    return dq, dk, dv


def fb_lowrank_mulbias_attn_fwd_workspace_bytes(B, H, N, C, R, dtype_code=FB_BF16) -> int:
    return int(load_library().fb_lowrank_mulbias_attn_fwd_workspace_bytes(B, H, N, C, R, dtype_code))


def fb_lowrank_mulbias_attn_fwd(q, k, v, phi_q, phi_k, out=None, lse=None, causal=False,
                                scale: float = 0.0, phi_batch_broadcast: Optional[bool] = None,
                                workspace=None, stream=None):
    """out, lse = softmax((q k^T scale) * (phi_q phi_k^T)) v, the multiplicative-bias form.
    q, k, v: [B,H,N,C] bf16; phi_q, phi_k: [B or 1,H,N,R], R >= 1, C (R - 1) <= 128 for C <= 64 (R = 1 at C = 128)."""
    lib = load_library()
    B, H, N, C = q.shape
    R = phi_q.shape[-1]
    if phi_batch_broadcast is None:
        phi_batch_broadcast = phi_q.shape[0] == 1 and B > 1
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    need = fb_lowrank_mulbias_attn_fwd_workspace_bytes(B, H, N, C, R)
    if workspace is None:
        workspace = _scratch(need, q.device, stream)
    st = lib.fb_lowrank_mulbias_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(phi_q), _ptr(phi_k), _ptr(out),
                                         _ptr(lse), B, H, N, C, R, int(bool(causal)), _dtype_code(q),
                                         _dtype_code(phi_q), int(bool(phi_batch_broadcast)), float(scale),
                                         _ptr(workspace), workspace.numel(), _stream(stream))
    _check(st, "fb_lowrank_mulbias_attn_fwd")
    return out, lse


def fb_lowrank_mulbias_attn_bwd_workspace_bytes(B, H, N, C, R, dtype_code=FB_BF16) -> int:
    return int(load_library().fb_lowrank_mulbias_attn_bwd_workspace_bytes(B, H, N, C, R, dtype_code))


def fb_lowrank_mulbias_attn_bwd(q, k, v, phi_q, phi_k, out, lse, dout, causal=False, scale: float = 0.0,
                                phi_batch_broadcast: Optional[bool] = None, workspace=None, grads=None,
                                stream=None):
    """dq, dk, dv, dphi_q, dphi_k of the multiplicative-bias attention (dphi_*: [B,H,N,R] in the
    factors' dtype, per batch element)."""
    lib = load_library()
    B, H, N, C = q.shape
    R = phi_q.shape[-1]
    if phi_batch_broadcast is None:
        phi_batch_broadcast = phi_q.shape[0] == 1 and B > 1
    need = fb_lowrank_mulbias_attn_bwd_workspace_bytes(B, H, N, C, R)
    if workspace is None:
        workspace = _scratch(need, q.device, stream)
    if grads is None:
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        dpq = torch.empty((B, H, N, R), dtype=phi_q.dtype, device=q.device)
        dpk = torch.empty((B, H, N, R), dtype=phi_k.dtype, device=q.device)
    else:
        dq, dk, dv, dpq, dpk = grads
    st = lib.fb_lowrank_mulbias_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(phi_q), _ptr(phi_k), _ptr(out), _ptr(lse),
                                         _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dpq), _ptr(dpk),
                                         B, H, N, C, R, int(bool(causal)), _dtype_code(q), _dtype_code(phi_q),
                                         int(bool(phi_batch_broadcast)), float(scale), _ptr(workspace),
                                         workspace.numel(), _stream(stream))
    _check(st, "fb_lowrank_mulbias_attn_bwd")
    return dq, dk, dv, dpq, dpk


def fb_alibi_attn_fwd(q, k, v, slopes, out=None, lse=None, causal=False, scale: float = 0.0,
                      stream=None):
    """out, lse = attention(q, k, v) with the bias -slopes[h] * (i - j) generated in the kernel.
    slopes: [H] float32 CUDA tensor."""
    lib = load_library()
    B, H, N, C = q.shape
    if slopes.dtype != torch.float32 or slopes.numel() != H:
        raise FlashBiasError("slopes must be a float32 tensor with one entry per head")
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    st = lib.fb_alibi_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(slopes), _ptr(out), _ptr(lse),
                               B, H, N, C, int(bool(causal)), _dtype_code(q), float(scale),
                               _stream(stream))
    _check(st, "fb_alibi_attn_fwd")
    return out, lse


def fb_dense_bias_attn_fwd(q, k, v, bias, out=None, lse=None, causal=False, scale: float = 0.0,
                           bias_batch_broadcast: Optional[bool] = None, stream=None):
    """out, lse = attention(q, k, v) with a dense bias [B or 1,H,N,N] of q's dtype."""
    lib = load_library()
    B, H, N, C = q.shape
    if bias_batch_broadcast is None:
        bias_batch_broadcast = bias.shape[0] == 1 and B > 1
    if bias.dtype != q.dtype:
        raise FlashBiasError("dense bias must have q's dtype")
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    st = lib.fb_dense_bias_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(bias), _ptr(out), _ptr(lse),
                                    B, H, N, C, int(bool(causal)), _dtype_code(q),
                                    int(bool(bias_batch_broadcast)), float(scale), _stream(stream))
    _check(st, "fb_dense_bias_attn_fwd")
    return out, lse


def fb_lowrank_attn_bwd_workspace_bytes(B, H, N, C, R, dtype_code=FB_BF16) -> int:
    return int(load_library().fb_lowrank_attn_bwd_workspace_bytes(B, H, N, C, R, dtype_code))


def fb_lowrank_attn_bwd(q, k, v, phi_q, phi_k, out, lse, dout, causal=False, scale: float = 0.0,
                        phi_batch_broadcast: Optional[bool] = None, workspace=None, grads=None,
                        stream=None):
    """dq, dk, dv, dphi_q, dphi_k for an upstream gradient dout.  dphi_* are [B,H,N,R]
    (per batch element) in the factors' dtype; None when R = 0."""
    lib = load_library()
    B, H, N, C = q.shape
    R = 0 if phi_q is None else phi_q.shape[-1]
    if phi_batch_broadcast is None:
        phi_batch_broadcast = phi_q is not None and phi_q.shape[0] == 1 and B > 1
    phi_code = _dtype_code(phi_q) if phi_q is not None else _dtype_code(q)
    need = fb_lowrank_attn_bwd_workspace_bytes(B, H, N, C, R, _dtype_code(q))
    if workspace is None:
        workspace = _scratch(need, q.device, stream)
    if grads is None:
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        dpq = dpk = None
        if R:
            dpq = torch.empty((B, H, N, R), dtype=phi_q.dtype, device=q.device)
            dpk = torch.empty((B, H, N, R), dtype=phi_q.dtype, device=q.device)
    else:
        dq, dk, dv, dpq, dpk = grads
    st = lib.fb_lowrank_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(phi_q), _ptr(phi_k), _ptr(out),
                                 _ptr(lse), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dpq),
                                 _ptr(dpk), B, H, N, C, R, int(bool(causal)), _dtype_code(q),
                                 phi_code, int(bool(phi_batch_broadcast)), float(scale),
                                 _ptr(workspace), workspace.numel() * workspace.element_size(),
                                 _stream(stream))
    _check(st, "fb_lowrank_attn_bwd")
    return dq, dk, dv, dpq, dpk


def fb_lowrank_attn_bwd_noalloc(q, k, v, phi_q, phi_k, out, lse, dout, grads, causal=False, scale: float = 0.0,
                                phi_batch_broadcast: Optional[bool] = None, stream=None):
    """fb_lowrank_attn_bwd on the library's static scratch: the caller passes every output tensor
    (grads = (dq, dk, dv, dphi_q, dphi_k); the last two None when R = 0 or not wanted) and this
    wrapper allocates nothing either."""
    lib = load_library()
    B, H, N, C = q.shape
    R = 0 if phi_q is None else phi_q.shape[-1]
    if phi_batch_broadcast is None:
        phi_batch_broadcast = phi_q is not None and phi_q.shape[0] == 1 and B > 1
    phi_code = _dtype_code(phi_q) if phi_q is not None else _dtype_code(q)
    dq, dk, dv, dpq, dpk = grads
    st = lib.fb_lowrank_attn_bwd_noalloc(_ptr(q), _ptr(k), _ptr(v), _ptr(phi_q), _ptr(phi_k), _ptr(out),
                                         _ptr(lse), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dpq),
                                         _ptr(dpk), B, H, N, C, R, int(bool(causal)), _dtype_code(q),
                                         phi_code, int(bool(phi_batch_broadcast)), float(scale),
                                         _stream(stream))
    _check(st, "fb_lowrank_attn_bwd_noalloc")
    return dq, dk, dv, dpq, dpk


def fb_lowrank_xattn_bwd(q, k, v, phi_q, phi_k, out, lse, dout, scale: float = 0.0,
                         phi_batch_broadcast: Optional[bool] = None, workspace=None, stream=None):
    """Cross-attention backward: returns dq [B,H,N,C], dk, dv [B,H,M,C], dphi_q [B,H,N,R],
    dphi_k [B,H,M,R] (None when R = 0)."""
    lib = load_library()
    B, H, N, C = q.shape
    M = k.shape[2]
    R = 0 if phi_q is None else phi_q.shape[-1]
    if phi_batch_broadcast is None:
        phi_batch_broadcast = phi_q is not None and phi_q.shape[0] == 1 and B > 1
    phi_code = _dtype_code(phi_q) if phi_q is not None else _dtype_code(q)
    need = int(lib.fb_lowrank_xattn_bwd_workspace_bytes(B, H, N, M, C, R, _dtype_code(q)))
    if workspace is None:
        workspace = _scratch(need, q.device, stream)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    dpq = dpk = None
    if R:
        dpq = torch.empty((B, H, N, R), dtype=phi_q.dtype, device=q.device)
        dpk = torch.empty((B, H, M, R), dtype=phi_q.dtype, device=q.device)
    st = lib.fb_lowrank_xattn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(phi_q), _ptr(phi_k), _ptr(out),
                                  _ptr(lse), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dpq),
                                  _ptr(dpk), B, H, N, M, C, R, _dtype_code(q), phi_code,
                                  int(bool(phi_batch_broadcast)), float(scale), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "fb_lowrank_xattn_bwd")
    return dq, dk, dv, dpq, dpk


def fb_dense_bias_attn_bwd_workspace_bytes(B, H, N, C, dtype_code=FB_BF16) -> int:
    return int(load_library().fb_dense_bias_attn_bwd_workspace_bytes(B, H, N, C, dtype_code))


def fb_lowrank_xattn_bwd_workspace_bytes(B, H, N, M, C, R, dtype_code=FB_BF16) -> int:
    return int(load_library().fb_lowrank_xattn_bwd_workspace_bytes(B, H, N, M, C, R, dtype_code))


def fb_dense_bias_attn_bwd(q, k, v, bias, out, lse, dout, causal=False, scale: float = 0.0,
                           bias_batch_broadcast: Optional[bool] = None, workspace=None, grads=None,
                           stream=None):
    """dq, dk, dv, dbias ([B,H,N,N], q's dtype) for the dense-bias attention."""
    lib = load_library()
    B, H, N, C = q.shape
    if bias_batch_broadcast is None:
        bias_batch_broadcast = bias.shape[0] == 1 and B > 1
    need = int(lib.fb_dense_bias_attn_bwd_workspace_bytes(B, H, N, C, _dtype_code(q)))
    if workspace is None:
        workspace = _scratch(need, q.device, stream)
    if grads is None:
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        dbias = torch.empty((B, H, N, N), dtype=q.dtype, device=q.device)
    else:
        dq, dk, dv, dbias = grads
    st = lib.fb_dense_bias_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(bias), _ptr(out), _ptr(lse),
                                    _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dbias),
                                    B, H, N, C, int(bool(causal)), _dtype_code(q),
                                    int(bool(bias_batch_broadcast)), float(scale), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "fb_dense_bias_attn_bwd")
    return dq, dk, dv, dbias
