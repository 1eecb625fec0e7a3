"""Differentiable wrappers: the library's forward and backward entry points as torch.autograd functions.

Training with factors (Sec. 3.2, "training" paragraph; Sec. 4.3): the factor tensors are ordinary
leaves of the graph and receive their gradients from the backward kernels, so an N x M bias
parameter can be replaced by N x R and M x R parameters (SVD type), by fixed exact factors, or by
the outputs of token-wise networks (neural type) without any other change to the model.

Nothing is computed here except what autograd's own bookkeeping needs: tensors are made
contiguous, the forward entry point is called, its inputs and (out, lse) are saved, and the
backward entry point is called on the upstream gradient.  The only arithmetic outside the
kernels is the chain rule of broadcasting: when factors (or a dense bias, or the ALiBi slopes)
are shared over the batch, the per-batch-element gradients the kernels return are summed over
the batch dimension with torch.sum.  There is no fallback path: without the shared library
every call raises.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import api


def _c(t: Optional[torch.Tensor]) -> Optional[torch.Tensor]:
    return None if t is None else t.contiguous()


def _fold_batch(g: Optional[torch.Tensor], like: Optional[torch.Tensor]) -> Optional[torch.Tensor]:
    """Gradient of a tensor that was broadcast over the batch: sum of the per-element gradients."""
    if g is None or like is None:
        return None
    if like.shape[0] == 1 and g.shape[0] > 1:
        return g.sum(dim=0, keepdim=True, dtype=torch.float32).to(like.dtype)
    return g


class _LowRank(torch.autograd.Function):
    """softmax(q k^T scale + phi_q phi_k^T) v (Eq. 3); N queries, M keys (causal needs N = M)."""

    @staticmethod
    def forward(ctx, q, k, v, phi_q, phi_k, causal, scale):
        q, k, v, phi_q, phi_k = _c(q), _c(k), _c(v), _c(phi_q), _c(phi_k)
        cross = q.shape[2] != k.shape[2]
        if cross:
            if causal:
                raise api.FlashBiasError("causal masking needs as many queries as keys")
            out, lse = api.fb_lowrank_xattn_fwd(q, k, v, phi_q, phi_k, scale=scale)
        else:
            out, lse = api.fb_lowrank_attn_fwd(q, k, v, phi_q, phi_k, causal=causal, scale=scale)
        ctx.save_for_backward(q, k, v, phi_q, phi_k, out, lse)
        ctx.cfg = (bool(causal), float(scale), cross)
        return out

    @staticmethod
    def backward(ctx, dout):
        q, k, v, phi_q, phi_k, out, lse = ctx.saved_tensors
        causal, scale, cross = ctx.cfg
        dout = _c(dout)
        if cross:
            dq, dk, dv, dpq, dpk = api.fb_lowrank_xattn_bwd(q, k, v, phi_q, phi_k, out, lse, dout, scale=scale)
        else:
            dq, dk, dv, dpq, dpk = api.fb_lowrank_attn_bwd(q, k, v, phi_q, phi_k, out, lse, dout,
                                                           causal=causal, scale=scale)
        return dq, dk, dv, _fold_batch(dpq, phi_q), _fold_batch(dpk, phi_k), None, None


class _MulBias(torch.autograd.Function):
    """softmax((q k^T scale) * (phi_q phi_k^T)) v (App. I)."""

    @staticmethod
    def forward(ctx, q, k, v, phi_q, phi_k, causal, scale):
        q, k, v, phi_q, phi_k = _c(q), _c(k), _c(v), _c(phi_q), _c(phi_k)
        out, lse = api.fb_lowrank_mulbias_attn_fwd(q, k, v, phi_q, phi_k, causal=causal, scale=scale)
        ctx.save_for_backward(q, k, v, phi_q, phi_k, out, lse)
        ctx.cfg = (bool(causal), float(scale))
        return out

    @staticmethod
    def backward(ctx, dout):
        q, k, v, phi_q, phi_k, out, lse = ctx.saved_tensors
        causal, scale = ctx.cfg
        dq, dk, dv, dpq, dpk = api.fb_lowrank_mulbias_attn_bwd(q, k, v, phi_q, phi_k, out, lse, _c(dout),
                                                               causal=causal, scale=scale)
        return dq, dk, dv, _fold_batch(dpq, phi_q), _fold_batch(dpk, phi_k), None, None


class _Alibi(torch.autograd.Function):
    """Bias -slopes[h] (i - j) generated inside the kernels (Example 3.4, App. D)."""

    @staticmethod
    def forward(ctx, q, k, v, slopes, causal, scale):
        q, k, v, slopes = _c(q), _c(k), _c(v), _c(slopes)
        out, lse = api.fb_alibi_attn_fwd(q, k, v, slopes, causal=causal, scale=scale)
        ctx.save_for_backward(q, k, v, slopes, out, lse)
        ctx.cfg = (bool(causal), float(scale))
        return out

    @staticmethod
    def backward(ctx, dout):
        q, k, v, slopes, out, lse = ctx.saved_tensors
        causal, scale = ctx.cfg
        rows = None
        if ctx.needs_input_grad[3]:
            rows = torch.empty(q.shape[:3], dtype=torch.float32, device=q.device)
        dq, dk, dv = api.fb_alibi_attn_bwd(q, k, v, slopes, out, lse, _c(dout), causal=causal, scale=scale,
                                           dslope_rows=rows)
        dslopes = None if rows is None else rows.sum(dim=(0, 2)).reshape(slopes.shape)
        return dq, dk, dv, dslopes, None, None


class _DenseBias(torch.autograd.Function):
    """The materialised-bias baseline (Eq. 1) with its N x N bias gradient (Sec. 4.3)."""

    @staticmethod
    def forward(ctx, q, k, v, bias, causal, scale):
        q, k, v, bias = _c(q), _c(k), _c(v), _c(bias)
        out, lse = api.fb_dense_bias_attn_fwd(q, k, v, bias, causal=causal, scale=scale)
        ctx.save_for_backward(q, k, v, bias, out, lse)
        ctx.cfg = (bool(causal), float(scale))
        return out

    @staticmethod
    def backward(ctx, dout):
        q, k, v, bias, out, lse = ctx.saved_tensors
        causal, scale = ctx.cfg
        dq, dk, dv, dbias = api.fb_dense_bias_attn_bwd(q, k, v, bias, out, lse, _c(dout), causal=causal,
                                                       scale=scale)
        return dq, dk, dv, _fold_batch(dbias, bias), None, None


def lowrank_bias_attention(q, k, v, phi_q=None, phi_k=None, causal: bool = False, scale: float = 0.0):
    """Attention with the additive bias phi_q phi_k^T.  q [B,H,N,C]; k, v [B,H,M,C]; phi_q [B or 1,H,N,R];
    phi_k [B or 1,H,M,R]; scale 0 means 1/sqrt(C).  Differentiable in q, k, v, phi_q, phi_k."""
    return _LowRank.apply(q, k, v, phi_q, phi_k, causal, scale)


def multiplicative_bias_attention(q, k, v, phi_q, phi_k, causal: bool = False, scale: float = 0.0):
    """Attention whose scores are multiplied by phi_q phi_k^T.  Differentiable in all five tensors."""
    return _MulBias.apply(q, k, v, phi_q, phi_k, causal, scale)


def alibi_attention(q, k, v, slopes, causal: bool = True, scale: float = 0.0):
    """Attention with the ALiBi bias -slopes[h] (i - j); slopes: [H] float32.  Differentiable in q, k, v, slopes."""
    return _Alibi.apply(q, k, v, slopes, causal, scale)


def dense_bias_attention(q, k, v, bias, causal: bool = False, scale: float = 0.0):
    """Attention with a materialised bias [B or 1,H,N,N] of q's dtype.  Differentiable in q, k, v, bias."""
    return _DenseBias.apply(q, k, v, bias, causal, scale)
