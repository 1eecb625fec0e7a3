"""The differentiable wrappers (paper_2505_12044_amd/autograd.py): what autograd delivers equals what
the backward entry points return, gradients of batch-shared tensors are the batch sums, parity with
the float64 oracle on a small case, and a short training run on factor parameters (Sec. 3.2,
training with factors: an N x M bias parameter replaced by N x R and M x R parameters)."""
import numpy as np
import pytest
import torch

from oracle import fb_oracle as O
from paper_2505_12044_amd import api, autograd as FA, workloads as W
from tests._gpu_util import check_fwd, check_grad, dev, host

pytestmark = pytest.mark.gpu


def _inputs(B, H, N, M, C, seed):
    rng = np.random.default_rng(seed)
    mk = lambda *s: W.round_bf16(rng.standard_normal(s).astype(np.float32))
    return mk(B, H, N, C), mk(B, H, M, C), mk(B, H, M, C), mk(B, H, N, C)


def _leaf(x, dtype="bf16"):
    return dev(x, dtype).requires_grad_(True)


@pytest.mark.parametrize("N,M,C,R,causal,phi_dtype,shared", [
    (200, 200, 64, 8, True, "bf16", False),
    (130, 130, 128, 2, False, "f32", True),
    (96, 160, 32, 16, False, "bf16", True),      # cross-attention
    (77, 77, 16, 0, True, "bf16", False),        # no bias
])
def test_lowrank_autograd_matches_entry_points_and_oracle(N, M, C, R, causal, phi_dtype, shared):
    B, H = 2, 3
    q, k, v, dout = _inputs(B, H, N, M, C, seed=9100 + N + C)
    rng = np.random.default_rng(9200 + R)
    Bp = 1 if shared else B
    pq = pk = None
    if R:
        pq = (0.4 * rng.standard_normal((Bp, H, N, R))).astype(np.float32)
        pk = (0.4 * rng.standard_normal((Bp, H, M, R))).astype(np.float32)
        if phi_dtype == "bf16":
            pq, pk = W.round_bf16(pq), W.round_bf16(pk)
    tq, tk, tv = _leaf(q), _leaf(k), _leaf(v)
    tpq = _leaf(pq, phi_dtype) if R else None
    tpk = _leaf(pk, phi_dtype) if R else None
    out = FA.lowrank_bias_attention(tq, tk, tv, tpq, tpk, causal=causal)
    tdo = dev(dout, "bf16")
    out.backward(tdo)
    torch.cuda.synchronize()

    # the same calls made by hand
    with torch.no_grad():
        if N == M:
            o2, lse = api.fb_lowrank_attn_fwd(tq, tk, tv, tpq, tpk, causal=causal)
            g = api.fb_lowrank_attn_bwd(tq, tk, tv, tpq, tpk, o2, lse, tdo, causal=causal)
        else:
            o2, lse = api.fb_lowrank_xattn_fwd(tq, tk, tv, tpq, tpk)
            g = api.fb_lowrank_xattn_bwd(tq, tk, tv, tpq, tpk, o2, lse, tdo)
    torch.cuda.synchronize()
    assert torch.equal(out.detach(), o2)
    for leaf, direct in zip((tq, tk, tv), g[:3]):
        assert torch.equal(leaf.grad, direct)
    if R:
        for leaf, direct in zip((tpq, tpk), g[3:]):
            assert leaf.grad.shape == leaf.shape and leaf.grad.dtype == leaf.dtype
            want = direct.sum(dim=0, keepdim=True, dtype=torch.float32).to(leaf.dtype) if shared else direct
            assert torch.equal(leaf.grad, want)

    # and against the oracle, one (b, h) at a time
    label = f"autograd lowrank N{N} M{M} C{C} R{R} causal={causal} {phi_dtype} shared={shared}"
    acc_pq = np.zeros((H, N, R)); acc_pk = np.zeros((H, M, R))
    for b in range(B):
        for h in range(H):
            bp = 0 if shared else b
            fq = pq[bp, h] if R else np.zeros((N, 0))
            fk = pk[bp, h] if R else np.zeros((M, 0))
            ro, _ = O.attention_lowrank(q[b, h], k[b, h], v[b, h], fq, fk, causal=causal)
            check_fwd(label, f"out[{b},{h}]", host(out[b, h]), ro)
            rg = O.attention_lowrank_grads(q[b, h], k[b, h], v[b, h], fq, fk, dout[b, h], causal=causal)
            for name, leaf, ref in (("dq", tq, rg[0]), ("dk", tk, rg[1]), ("dv", tv, rg[2])):
                check_grad(label, f"{name}[{b},{h}]", host(leaf.grad[b, h]), ref, data_scaled=True)
            if R and not shared:
                check_grad(label, f"dphi_q[{b},{h}]", host(tpq.grad[b, h]), rg[3], data_scaled=True)
                check_grad(label, f"dphi_k[{b},{h}]", host(tpk.grad[b, h]), rg[4], data_scaled=True)
            elif R:
                acc_pq[h] += rg[3]; acc_pk[h] += rg[4]
    if R and shared:
        check_grad(label, "dphi_q summed over the batch", host(tpq.grad[0]), acc_pq, data_scaled=True)
        check_grad(label, "dphi_k summed over the batch", host(tpk.grad[0]), acc_pk, data_scaled=True)


def test_alibi_dense_and_multiplicative_autograd_match_entry_points():
    B, H, N, C = 2, 4, 160, 64
    q, k, v, dout = _inputs(B, H, N, N, C, seed=9300)
    tdo = dev(dout, "bf16")

    # ALiBi in the kernel: dslopes is the sum of the per-row contributions
    slopes = torch.from_numpy(W.alibi_slopes_f32(H)).cuda().requires_grad_(True)
    tq, tk, tv = _leaf(q), _leaf(k), _leaf(v)
    out = FA.alibi_attention(tq, tk, tv, slopes, causal=True)
    out.backward(tdo)
    with torch.no_grad():
        o2, lse = api.fb_alibi_attn_fwd(tq, tk, tv, slopes, causal=True)
        rows = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
        g = api.fb_alibi_attn_bwd(tq, tk, tv, slopes, o2, lse, tdo, causal=True, dslope_rows=rows)
    torch.cuda.synchronize()
    assert torch.equal(out.detach(), o2)
    for leaf, direct in zip((tq, tk, tv), g):
        assert torch.equal(leaf.grad, direct)
    assert torch.equal(slopes.grad, rows.sum(dim=(0, 2)))
    # the slope gradient against the oracle's bias gradient: d slope_h = -sum_ij dB_ij (i - j)
    i = np.arange(N)
    dist = (i[:, None] - i[None, :]).astype(np.float64)
    for h in range(H):
        ref = 0.0
        for b in range(B):
            bias = -float(slopes.detach()[h]) * dist
            dS = O.attention_with_bias_grads(q[b, h], k[b, h], v[b, h], bias, dout[b, h], causal=True)[3]
            ref += float(np.sum(dS * -dist))
        got = float(slopes.grad[h])
        print(f"[parity] autograd alibi dslope[{h}]: got {got:.5g} ref {ref:.5g}", flush=True)
        assert abs(got - ref) <= 5e-2 * max(1.0, abs(ref))

    # dense bias shared over the batch: dbias is summed over the batch
    rng = np.random.default_rng(9301)
    bias = W.round_bf16((0.5 * rng.standard_normal((1, H, N, N))).astype(np.float32))
    tq, tk, tv, tb = _leaf(q), _leaf(k), _leaf(v), _leaf(bias)
    out = FA.dense_bias_attention(tq, tk, tv, tb, causal=False)
    out.backward(tdo)
    with torch.no_grad():
        o2, lse = api.fb_dense_bias_attn_fwd(tq, tk, tv, tb)
        g = api.fb_dense_bias_attn_bwd(tq, tk, tv, tb, o2, lse, tdo)
    torch.cuda.synchronize()
    assert torch.equal(out.detach(), o2)
    for leaf, direct in zip((tq, tk, tv), g[:3]):
        assert torch.equal(leaf.grad, direct)
    assert tb.grad.shape == tb.shape
    assert torch.equal(tb.grad, g[3].sum(dim=0, keepdim=True, dtype=torch.float32).to(torch.bfloat16))

    # multiplicative bias
    pq = (1.0 + 0.2 * rng.standard_normal((B, H, N, 2))).astype(np.float32)
    pk = (1.0 + 0.2 * rng.standard_normal((B, H, N, 2))).astype(np.float32)
    tq, tk, tv, tpq, tpk = _leaf(q), _leaf(k), _leaf(v), _leaf(pq, "f32"), _leaf(pk, "f32")
    out = FA.multiplicative_bias_attention(tq, tk, tv, tpq, tpk, causal=True)
    out.backward(tdo)
    with torch.no_grad():
        o2, lse = api.fb_lowrank_mulbias_attn_fwd(tq, tk, tv, tpq, tpk, causal=True)
        g = api.fb_lowrank_mulbias_attn_bwd(tq, tk, tv, tpq, tpk, o2, lse, tdo, causal=True)
    torch.cuda.synchronize()
    assert torch.equal(out.detach(), o2)
    for leaf, direct in zip((tq, tk, tv, tpq, tpk), g):
        assert torch.equal(leaf.grad, direct)


def test_training_factor_parameters_recovers_a_low_rank_bias():
    """SVD-type training: the attention's bias is phi_q phi_k^T with phi_q, phi_k free fp32 parameters
    (shared over the batch), fitted by Adam so that the layer's output matches the output produced with
    a hidden rank-4 bias.  q, k, v stay fixed; only gradients from the backward kernels drive the fit."""
    B, H, N, C, R = 4, 2, 256, 64, 4
    q, k, v, _ = _inputs(B, H, N, N, C, seed=9400)
    rng = np.random.default_rng(9401)
    hq = (0.8 * rng.standard_normal((1, H, N, R))).astype(np.float32)
    hk = (0.8 * rng.standard_normal((1, H, N, R))).astype(np.float32)
    tq, tk, tv = dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16")
    with torch.no_grad():
        target, _ = api.fb_lowrank_attn_fwd(tq, tk, tv, dev(hq, "f32"), dev(hk, "f32"))
        target = target.float()
    torch.manual_seed(0)
    pq = torch.nn.Parameter(0.1 * torch.randn(1, H, N, R, device="cuda"))
    pk = torch.nn.Parameter(0.1 * torch.randn(1, H, N, R, device="cuda"))
    opt = torch.optim.Adam([pq, pk], lr=5e-2)
    losses = []
    for step in range(300):
        opt.zero_grad(set_to_none=True)
        out = FA.lowrank_bias_attention(tq, tk, tv, pq, pk)
        loss = (out.float() - target).square().mean()
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    print(f"[train] loss {losses[0]:.4e} -> {losses[-1]:.4e}", flush=True)
    assert np.isfinite(losses).all()
    assert losses[-1] < 0.1 * losses[0]
    # the learned factors reproduce the hidden bias up to the softmax's row-constant freedom
    with torch.no_grad():
        bl = (pq[0].double() @ pk[0].double().transpose(-1, -2)).cpu().numpy()
    bh = np.einsum("hnr,hmr->hnm", hq[0].astype(np.float64), hk[0].astype(np.float64))
    dl = bl - bl.mean(axis=-1, keepdims=True)
    dh = bh - bh.mean(axis=-1, keepdims=True)
    rel = np.linalg.norm(dl - dh) / np.linalg.norm(dh)
    print(f"[train] relative distance of the learned bias (rows centred) to the hidden one: {rel:.3f}", flush=True)
    assert rel < 0.6
