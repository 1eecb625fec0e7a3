"""Float64 CPU oracle for attention with an additive bias (FlashBias, arxiv 2505.12044).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import it.  It shares no code, table, constant or
helper with the HIP kernels and never calls them.

What it computes is the plain definition the fast method must reproduce (Sec. 2.1, Eq. 1):

    o = softmax(q k^T / sqrt(C) + b) v,        q: N x C,  k, v: M x C,  b: N x M

with the bias either given densely or materialised from factors b = phi_q phi_k^T
(Sec. 3.2, Eq. 2).  Nothing is tiled, fused or rescaled on line: every score row is
formed whole, a two-pass softmax is taken over it, and the value product follows.  The
only concession to memory is that query rows may be processed a block of whole rows at
a time (rows of a softmax are independent, so this changes no arithmetic within a row;
key-side gradients are sums over query rows and are accumulated block by block).

Gradients are the chain rule applied to those same steps for the loss L = sum(dO * O).
The paper prints no backward formulas (it trains through a framework's autograd on the
concatenated operands, Sec. 4.1 "Implementation choices"); the derivation is the
textbook one and is pinned by finite differences in the CPU tests.

All arithmetic is numpy float64.  Inputs are converted with np.asarray(x, float64), so a
caller that wants "what the kernel saw" passes values already rounded to the kernel's
storage type.

Parity pins (tests/test_oracle_pins.py): exact ALiBi rank-2 factorisation (Example 3.4),
the rank-9 squared-distance factorisation (Example 3.5), the channel-concatenation
identity (Eq. 3), closed forms for q = 0, softmax invariants, a library cross-check
against torch's float64 scaled_dot_product_attention, Eckart-Young for truncated SVD
(Remark 3.8's "energy"), and central finite differences plus invariants for gradients.
The batched wrappers are pinned slice by slice against the single-head functions and, as whole
[B,H,N,.] tensors, against torch float64 autograd / scaled_dot_product_attention with shared
factors or bias as one broadcast parameter.
The paper prints no worked numeric example of attention outputs, so output values are
pinned only through those identities, closed forms and the library cross-check.

The multiplicative-bias extension (App. I) is covered by its definition
o = softmax((q k^T / sqrt(C)) o b) v with b materialised, pinned by brute force on tiny
inputs, by b = 1 reducing to plain attention, by the cos(i - j) rank-2 example and by the
repeated-and-reweighted-channel identity of that appendix.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "lowrank_bias",
    "attention_with_bias",
    "attention_lowrank",
    "attention_with_multiplicative_bias",
    "attention_multiplicative_lowrank_grads",
    "multiplicative_concat",
    "cosine_multiplicative_factors",
    "attention_with_bias_grads",
    "attention_lowrank_grads",
    "batched_attention_lowrank",
    "batched_attention_dense",
    "batched_attention_lowrank_grads",
    "alibi_bias",
    "alibi_slopes",
    "squared_distance_bias",
    "squared_distance_factors",
    "truncated_svd_factors",
    "svd_energy",
    "hbm_io_ratio_example",
]


def _f64(x):
    return np.asarray(x, dtype=np.float64)


# ----------------------------------------------------------------------------------
# Bias from factors (Sec. 3.2, Eq. 2)
# ----------------------------------------------------------------------------------
def lowrank_bias(phi_q, phi_k):
    """b = phi_q phi_k^T, materialised.  phi_q: N x R, phi_k: M x R.  R = 0 gives zeros."""
    phi_q = _f64(phi_q)
    phi_k = _f64(phi_k)
    if phi_q.shape[-1] == 0:
        return np.zeros((phi_q.shape[0], phi_k.shape[0]), dtype=np.float64)
    return phi_q @ phi_k.T


# ----------------------------------------------------------------------------------
# Forward (Sec. 2.1, Eq. 1)
# ----------------------------------------------------------------------------------
def _scores(q, k, bias, scale, causal, row_offset):
    """s = scale * q k^T + b, with entries above the diagonal set to -inf when causal.

    row_offset is the absolute index of q's first row, so a slice of query rows is masked
    exactly as it would be inside the full problem (key j is visible to query i iff j <= i).
    """
    s = scale * (q @ k.T)
    if bias is not None:
        s = s + bias
    if causal:
        i = np.arange(q.shape[0])[:, None] + row_offset
        j = np.arange(k.shape[0])[None, :]
        s = np.where(j > i, -np.inf, s)
    return s


def _softmax_rows(s):
    """Two-pass softmax over each whole row; also the natural-log log-sum-exp of the row."""
    m = np.max(s, axis=1, keepdims=True)
    e = np.exp(s - m)
    z = np.sum(e, axis=1, keepdims=True)
    p = e / z
    lse = (m + np.log(z))[:, 0]
    return p, lse


def attention_with_bias(q, k, v, bias=None, causal=False, scale=None, row_offset=0,
                        return_probs=False):
    """o = softmax(scale q k^T + b [+ causal mask]) v for one head.

    q: N x C, k, v: M x C, bias: N x M or None.  scale defaults to 1/sqrt(C).
    Returns (o [N x C], lse [N]) and additionally p [N x M] if return_probs.
    """
    q, k, v = _f64(q), _f64(k), _f64(v)
    if bias is not None:
        bias = _f64(bias)
    if scale is None:
        scale = 1.0 / np.sqrt(q.shape[1])
    s = _scores(q, k, bias, scale, causal, row_offset)
    p, lse = _softmax_rows(s)
    o = p @ v
    if return_probs:
        return o, lse, p
    return o, lse


def attention_lowrank(q, k, v, phi_q, phi_k, causal=False, scale=None, row_offset=0):
    """Same as attention_with_bias with b = phi_q phi_k^T materialised first (Eq. 2)."""
    b = lowrank_bias(phi_q, phi_k)
    return attention_with_bias(q, k, v, b, causal=causal, scale=scale, row_offset=row_offset)


# ----------------------------------------------------------------------------------
# Multiplicative bias (App. I)
# ----------------------------------------------------------------------------------
def attention_with_multiplicative_bias(q, k, v, b, causal=False, scale=None, row_offset=0):
    """o = softmax((scale q k^T) o b [+ causal mask]) v for one head, o = Hadamard product
    (App. I, the definition the extension starts from).  b: N x M dense.  scale defaults to
    1/sqrt(C) with C the channel count of q itself.  Returns (o, lse)."""
    q, k, v, b = _f64(q), _f64(k), _f64(v), _f64(b)
    if scale is None:
        scale = 1.0 / np.sqrt(q.shape[1])
    s = (scale * (q @ k.T)) * b
    if causal:
        i = np.arange(q.shape[0])[:, None] + row_offset
        j = np.arange(k.shape[0])[None, :]
        s = np.where(j > i, -np.inf, s)
    p, lse = _softmax_rows(s)
    return p @ v, lse


def multiplicative_concat(x, phi):
    """App. I's reweighted repeat: [x o phi_1, ..., x o phi_R] along the channel axis, each
    factor column broadcast over the C channels of x.  x: N x C, phi: N x R -> N x (C R)."""
    x, phi = _f64(x), _f64(phi)
    return np.concatenate([x * phi[:, r:r + 1] for r in range(phi.shape[1])], axis=1)


def cosine_multiplicative_factors(n, m=None):
    """App. I's example: b_ij = cos(i - j) = cos i cos j + sin i sin j, rank 2 (0-based positions)."""
    m = n if m is None else m
    i = np.arange(n, dtype=np.float64)
    j = np.arange(m, dtype=np.float64)
    return np.stack([np.cos(i), np.sin(i)], axis=1), np.stack([np.cos(j), np.sin(j)], axis=1)


# ----------------------------------------------------------------------------------
# Backward: chain rule through the steps above for L = sum(dO * O)
# ----------------------------------------------------------------------------------
def _grads_rows(q, k, v, bias, dout, causal, scale, row_offset):
    """Gradients contributed by a block of whole query rows.

    Returns dq (for these rows), the rows' contributions to dk and dv, and ds = dL/ds
    for these rows (which is also dL/db)."""
    s = _scores(q, k, bias, scale, causal, row_offset)
    p, _ = _softmax_rows(s)
    dv = p.T @ dout                      # o = p v
    dp = dout @ v.T
    # softmax Jacobian: ds_ij = p_ij (dp_ij - sum_l p_il dp_il)
    ds = p * (dp - np.sum(p * dp, axis=1, keepdims=True))
    dq = scale * (ds @ k)                # s = scale q k^T + b
    dk = scale * (ds.T @ q)
    return dq, dk, dv, ds


def attention_with_bias_grads(q, k, v, bias, dout, causal=False, scale=None):
    """(dq, dk, dv, dbias) for one head with a dense bias (dbias = dL/ds, N x M)."""
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    bias = None if bias is None else _f64(bias)
    if scale is None:
        scale = 1.0 / np.sqrt(q.shape[1])
    return _grads_rows(q, k, v, bias, dout, causal, scale, 0)


def attention_lowrank_grads(q, k, v, phi_q, phi_k, dout, causal=False, scale=None,
                            row_block=None):
    """(dq, dk, dv, dphi_q, dphi_k) for one head with b = phi_q phi_k^T.

    b = phi_q phi_k^T  =>  dphi_q = db phi_k,  dphi_k = db^T phi_q,  with db = ds.
    row_block bounds memory by taking whole query rows a block at a time.
    """
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    phi_q, phi_k = _f64(phi_q), _f64(phi_k)
    n, m = q.shape[0], k.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(q.shape[1])
    if row_block is None:
        row_block = n
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    dphi_q = np.zeros_like(phi_q)
    dphi_k = np.zeros_like(phi_k)
    for r0 in range(0, n, row_block):
        r1 = min(n, r0 + row_block)
        b = lowrank_bias(phi_q[r0:r1], phi_k)
        dq_r, dk_r, dv_r, ds = _grads_rows(q[r0:r1], k, v, b, dout[r0:r1], causal, scale, r0)
        dq[r0:r1] = dq_r
        dk += dk_r
        dv += dv_r
        if phi_q.shape[1]:
            dphi_q[r0:r1] = ds @ phi_k
            dphi_k += ds.T @ phi_q[r0:r1]
    return dq, dk, dv, dphi_q, dphi_k


def attention_multiplicative_lowrank_grads(q, k, v, phi_q, phi_k, dout, causal=False, scale=None):
    """(dq, dk, dv, dphi_q, dphi_k) for one head of the multiplicative form (App. I),
    s = (scale q k^T) o b with b = phi_q phi_k^T, L = sum(dO * O).  Chain rule on the definition
    (the appendix gives no backward): with a = scale q k^T and ds from the softmax Jacobian,
    da = ds o b, db = ds o a, dq = scale da k, dk = scale da^T q, dphi_q = db phi_k,
    dphi_k = db^T phi_q, dv = p^T dO."""
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    phi_q, phi_k = _f64(phi_q), _f64(phi_k)
    if scale is None:
        scale = 1.0 / np.sqrt(q.shape[1])
    b = phi_q @ phi_k.T
    a = scale * (q @ k.T)
    s = a * b
    if causal:
        i = np.arange(q.shape[0])[:, None]
        j = np.arange(k.shape[0])[None, :]
        s = np.where(j > i, -np.inf, s)
    p, _ = _softmax_rows(s)
    dv = p.T @ dout
    dp = dout @ v.T
    ds = p * (dp - np.sum(p * dp, axis=1, keepdims=True))
    da = ds * b
    db = ds * a
    return scale * (da @ k), scale * (da.T @ q), dv, db @ phi_k, db.T @ phi_q


# ----------------------------------------------------------------------------------
# Batched wrappers: [B, H, N, .] layouts; factor / bias tensors may have batch size 1
# ----------------------------------------------------------------------------------
def _bsel(x, b):
    return x[0 if x.shape[0] == 1 else b]


def batched_attention_lowrank(q, k, v, phi_q, phi_k, causal=False, scale=None):
    """q, k, v: [B,H,N,C]; phi_q, phi_k: [B or 1,H,N,R].  Returns out [B,H,N,C], lse [B,H,N]."""
    B, H, N, C = q.shape
    out = np.empty((B, H, N, C), dtype=np.float64)
    lse = np.empty((B, H, N), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            out[b, h], lse[b, h] = attention_lowrank(
                q[b, h], k[b, h], v[b, h], _bsel(phi_q, b)[h], _bsel(phi_k, b)[h],
                causal=causal, scale=scale)
    return out, lse


def batched_attention_dense(q, k, v, bias, causal=False, scale=None):
    """q, k, v: [B,H,N,C]; bias: [B or 1,H,N,N].  Returns out, lse."""
    B, H, N, C = q.shape
    out = np.empty((B, H, N, C), dtype=np.float64)
    lse = np.empty((B, H, N), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            out[b, h], lse[b, h] = attention_with_bias(
                q[b, h], k[b, h], v[b, h], _bsel(bias, b)[h], causal=causal, scale=scale)
    return out, lse


def batched_attention_lowrank_grads(q, k, v, phi_q, phi_k, dout, causal=False, scale=None,
                                    row_block=None):
    """Per-(b,h) gradients; dphi_q, dphi_k are returned per batch element ([B,H,N,R])
    even when the factors are shared over the batch (a caller sums over b for a shared
    parameter)."""
    B, H, N, C = q.shape
    R = phi_q.shape[-1]
    dq = np.empty((B, H, N, C)); dk = np.empty((B, H, N, C)); dv = np.empty((B, H, N, C))
    dpq = np.empty((B, H, N, R)); dpk = np.empty((B, H, N, R))
    for b in range(B):
        for h in range(H):
            dq[b, h], dk[b, h], dv[b, h], dpq[b, h], dpk[b, h] = attention_lowrank_grads(
                q[b, h], k[b, h], v[b, h], _bsel(phi_q, b)[h], _bsel(phi_k, b)[h], dout[b, h],
                causal=causal, scale=scale, row_block=row_block)
    return dq, dk, dv, dpq, dpk


# ----------------------------------------------------------------------------------
# Bias families the paper decomposes (Sec. 3.2).  These are the DENSE definitions and
# the paper's printed factorisations, used to pin the input generators.
# ----------------------------------------------------------------------------------
def alibi_slopes(num_heads):
    """Head slopes m_h = 2^(-8 (h+1) / num_heads), h = 0..num_heads-1 (the geometric
    sequence of the ALiBi scheme the paper's Example 3.4 refers to)."""
    h = np.arange(num_heads, dtype=np.float64)
    return 2.0 ** (-8.0 * (h + 1.0) / num_heads)


def alibi_bias(slope, n, m=None):
    """Dense ALiBi bias b_ij = -slope * (i - j), 0-based, for every (i, j); the causal mask
    is applied separately (Example 3.4 treats only the bias term)."""
    m = n if m is None else m
    i = np.arange(n, dtype=np.float64)[:, None]
    j = np.arange(m, dtype=np.float64)[None, :]
    return -slope * (i - j)


def squared_distance_bias(x_q, x_k):
    """b_ij = ||x_q,i - x_k,j||_2^2 written out as a double loop-free definition."""
    x_q, x_k = _f64(x_q), _f64(x_k)
    d = x_q[:, None, :] - x_k[None, :, :]
    return np.sum(d * d, axis=2)


def squared_distance_factors(x_q, x_k):
    """The rank-9 factors of Example 3.5 for 3-D positions, in the printed column order:
    phi_q(x) = [x0^2, 1, -2 x0, x1^2, 1, -2 x1, x2^2, 1, -2 x2],
    phi_k(y) = [1, y0^2, y0,   1, y1^2, y1,   1, y2^2, y2]."""
    x_q, x_k = _f64(x_q), _f64(x_k)
    one_q = np.ones(x_q.shape[0]); one_k = np.ones(x_k.shape[0])
    pq, pk = [], []
    for a in range(3):
        pq += [x_q[:, a] ** 2, one_q, -2.0 * x_q[:, a]]
        pk += [one_k, x_k[:, a] ** 2, x_k[:, a]]
    return np.stack(pq, axis=1), np.stack(pk, axis=1)


def truncated_svd_factors(bias, rank):
    """Rank-R factors of a dense N x M bias by truncated SVD (Sec. 3.2 "SVD decomposition"):
    bias ~= U_R S_R V_R^T with phi_q = U_R S_R^(1/2), phi_k = V_R S_R^(1/2).  The paper
    does not say how S is shared between the factors; the symmetric split is this
    build's reading and does not change phi_q phi_k^T."""
    u, s, vt = np.linalg.svd(_f64(bias), full_matrices=False)
    r = int(rank)
    root = np.sqrt(s[:r])
    return u[:, :r] * root[None, :], vt[:r, :].T * root[None, :]


def svd_energy(bias, rank):
    """Share of squared singular values kept by the leading `rank` of them (the reading of
    "energy" in Remark 3.8)."""
    s = np.linalg.svd(_f64(bias), compute_uv=False)
    return float(np.sum(s[: int(rank)] ** 2) / np.sum(s ** 2))


# ----------------------------------------------------------------------------------
# The HBM-traffic example (Example 3.9 and its calculation in Appendix A)
# ----------------------------------------------------------------------------------
def hbm_io_ratio_example(C=64, R=64, sram_bytes=100 * 1024, bytes_per_elem=2):
    """Ratio of HBM access, fused attention reading a dense bias over the factorised form,
    for N, M >> C, R:  (C^2/S + 1) * S / (C^2 + R^2)  with S counted in elements of
    `bytes_per_elem` bytes — the expression in the appendix evaluates this at C = R = 64,
    S = 100 KB, half precision."""
    c2 = bytes_per_elem * C * C
    r2 = bytes_per_elem * R * R
    return (1.0 + c2 / sram_bytes) * sram_bytes / (c2 + r2)
