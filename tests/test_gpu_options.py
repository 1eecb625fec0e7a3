"""GPU parity of the call options the other parity tests leave at their defaults: an explicit
softmax scale (Eq. 1's 1/sqrt(C) replaced by the caller's value) through every entry point and
forward kernel variant, a caller-supplied stream, caller-supplied output buffers, and the
binding's rejection of tensors it cannot pass on."""
import numpy as np
import pytest
import torch

from oracle import fb_oracle as O
from paper_2505_12044_amd import api, workloads as W
from tests._gpu_util import GRAD_TOL, TOL, dev, host, max_abs

pytestmark = pytest.mark.gpu


def _case(B, H, N, C, R, seed, phi_dtype="bf16"):
    rng = np.random.default_rng(seed)
    rd = lambda *s: W.round_bf16(rng.standard_normal(s).astype(np.float32))
    q, k, v, dout = rd(B, H, N, C), rd(B, H, N, C), rd(B, H, N, C), rd(B, H, N, C)
    pq = (R ** -0.25 * rng.standard_normal((B, H, N, R))).astype(np.float32)
    pk = (R ** -0.25 * rng.standard_normal((B, H, N, R))).astype(np.float32)
    if phi_dtype == "bf16":
        pq, pk = W.round_bf16(pq), W.round_bf16(pk)
    return q, k, v, dout, pq, pk


@pytest.mark.parametrize("factor", [0.4, 1.7])
@pytest.mark.parametrize("C", [16, 64, 128])
def test_explicit_scale_forward_variants(C, factor):
    # scale relative to the default: the score spread (and with it the absolute effect of the bf16
    # operand rounding, ~|s| 2^-9) stays in the range the 2e-2 bound is stated for
    scale = factor / np.sqrt(C)
    B, H, N, R = 1, 2, 300, 8
    q, k, v, _, pq, pk = _case(B, H, N, C, R, seed=9000 + C)
    d = [dev(x, "bf16") for x in (q, k, v, pq, pk)]
    ref = [O.attention_lowrank(q[0, h], k[0, h], v[0, h], pq[0, h], pk[0, h], causal=True, scale=scale)
           for h in range(H)]
    for qb in (1, 2, 8, 16):
        api.fb_tune_set("fwd_qb", qb)
        try:
            out, lse = api.fb_lowrank_attn_fwd(*d, causal=True, scale=scale)
            torch.cuda.synchronize()
        finally:
            api.fb_tune_set("fwd_qb", 0)
        eo = max(max_abs(host(out[0, h]), ref[h][0]) for h in range(H))
        el = max(max_abs(host(lse[0, h]), ref[h][1]) for h in range(H))
        print(f"scale {scale:.4f} C{C} qb={qb}: out {eo:.3e} lse {el:.3e}", flush=True)
        assert eo <= TOL["bf16"] and el <= TOL["bf16"]


@pytest.mark.parametrize("scale", [0.04, 0.2])
def test_explicit_scale_other_entry_points(scale):
    B, H, N, C, R = 1, 2, 264, 64, 4
    q, k, v, dout, pq, pk = _case(B, H, N, C, R, seed=9100, phi_dtype="f32")
    # fp32 forward
    f = [dev(x, "f32") for x in (q, k, v, pq, pk)]
    out, lse = api.fb_lowrank_attn_fwd(*f, scale=scale)
    torch.cuda.synchronize()
    for h in range(H):
        ro, rl = O.attention_lowrank(q[0, h], k[0, h], v[0, h], pq[0, h], pk[0, h], scale=scale)
        assert max_abs(host(out[0, h]), ro) <= TOL["f32"] and max_abs(host(lse[0, h]), rl) <= TOL["f32"]
    # dense forward + backward, low-rank backward (bf16)
    bias = W.round_bf16(np.einsum("bhir,bhjr->bhij", pq, pk).astype(np.float32))
    dq_, dk_, dv_, dd = dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), dev(dout, "bf16")
    db = dev(bias, "bf16")
    o2, l2 = api.fb_dense_bias_attn_fwd(dq_, dk_, dv_, db, scale=scale)
    g2 = api.fb_dense_bias_attn_bwd(dq_, dk_, dv_, db, o2, l2, dd, scale=scale)
    dpq, dpk = dev(pq, "f32"), dev(pk, "f32")
    o3, l3 = api.fb_lowrank_attn_fwd(dq_, dk_, dv_, dpq, dpk, scale=scale)
    g3 = api.fb_lowrank_attn_bwd(dq_, dk_, dv_, dpq, dpk, o3, l3, dd, scale=scale)
    torch.cuda.synchronize()
    worst = 0.0
    for h in range(H):
        ro, rl = O.attention_with_bias(q[0, h], k[0, h], v[0, h], bias[0, h], scale=scale)
        assert max_abs(host(o2[0, h]), ro) <= TOL["bf16"] and max_abs(host(l2[0, h]), rl) <= TOL["bf16"]
        rg = O.attention_with_bias_grads(q[0, h], k[0, h], v[0, h], bias[0, h], dout[0, h], scale=scale)
        for g, r in zip(g2, rg):
            worst = max(worst, max_abs(host(g[0, h]), r) / max(1.0, float(np.abs(r).max()) / 2.5))
        rg = O.attention_lowrank_grads(q[0, h], k[0, h], v[0, h], pq[0, h], pk[0, h], dout[0, h], scale=scale)
        for g, r in zip(g3, rg):
            worst = max(worst, max_abs(host(g[0, h]), r) / max(1.0, float(np.abs(r).max()) / 2.5))
    print(f"scale {scale}: worst scaled gradient err {worst:.3e}", flush=True)
    assert worst <= GRAD_TOL
    # cross-attention and the multiplicative form
    M = 200
    o4, l4 = api.fb_lowrank_xattn_fwd(dq_, dk_[:, :, :M].contiguous(), dv_[:, :, :M].contiguous(), dpq,
                                      dpk[:, :, :M].contiguous(), scale=scale)
    fq = np.clip(pq[..., :2], -1, 1); fk = np.clip(pk[..., :2], -1, 1)
    o5, l5 = api.fb_lowrank_mulbias_attn_fwd(dq_, dk_, dv_, dev(fq, "f32"), dev(fk, "f32"), scale=scale)
    torch.cuda.synchronize()
    for h in range(H):
        ro, rl = O.attention_lowrank(q[0, h], k[0, h, :M], v[0, h, :M], pq[0, h], pk[0, h, :M], scale=scale)
        assert max_abs(host(o4[0, h]), ro) <= TOL["bf16"] and max_abs(host(l4[0, h]), rl) <= TOL["bf16"]
        ro, rl = O.attention_with_multiplicative_bias(q[0, h], k[0, h], v[0, h],
                                                      O.lowrank_bias(fq[0, h], fk[0, h]), scale=scale)
        assert max_abs(host(o5[0, h]), ro) <= TOL["bf16"] and max_abs(host(l5[0, h]), rl) <= TOL["bf16"]


def test_alibi_explicit_scale():
    B, H, N, C = 1, 3, 333, 64
    q, k, v, _, _, _ = _case(B, H, N, C, 1, seed=9200)
    slopes = np.array([0.25, 0.03125, 0.007], dtype=np.float32)
    out, lse = api.fb_alibi_attn_fwd(dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"),
                                     torch.from_numpy(slopes).cuda(), causal=True, scale=0.2)
    torch.cuda.synchronize()
    for h in range(H):
        ro, rl = O.attention_with_bias(q[0, h], k[0, h], v[0, h], O.alibi_bias(float(slopes[h]), N),
                                       causal=True, scale=0.2)
        assert max_abs(host(out[0, h]), ro) <= TOL["bf16"] and max_abs(host(lse[0, h]), rl) <= TOL["bf16"]


@pytest.mark.parametrize("C,R,phi_dtype,causal", [(128, 2, "f32", True), (128, 8, "bf16", False), (64, 5, "f32", False),
                                                  (64, 16, "bf16", True)])
def test_power_of_two_scale_backward(C, R, phi_dtype, causal):
    """With a scale that is a power of two the backward reads q in place and carries 1/scale on the
    query-side factor columns instead (exact then); every gradient against the oracle, and the same
    call with a neighbouring scale that takes the other route."""
    B, H, N = 2, 2, 300
    q, k, v, dout, pq, pk = _case(B, H, N, C, R, seed=9500 + C + R, phi_dtype=phi_dtype)
    d = [dev(x, "bf16") for x in (q, k, v)] + [dev(pq, phi_dtype), dev(pk, phi_dtype)]
    dd = dev(dout, "bf16")
    for scale in (0.125, 0.11):
        out, lse = api.fb_lowrank_attn_fwd(*d, causal=causal, scale=scale)
        g = api.fb_lowrank_attn_bwd(*d, out, lse, dd, causal=causal, scale=scale)
        torch.cuda.synchronize()
        for b in range(B):
            for h in range(H):
                rg = O.attention_lowrank_grads(q[b, h], k[b, h], v[b, h], pq[b, h], pk[b, h], dout[b, h],
                                               causal=causal, scale=scale)
                for name, got, ref in zip(("dq", "dk", "dv", "dphi_q", "dphi_k"), g, rg):
                    e = max_abs(host(got[b, h]), ref)
                    lim = GRAD_TOL * max(1.0, float(np.abs(ref).max()) / 2.5)
                    print(f"[parity] scale {scale} C{C} R{R} {phi_dtype} causal={causal} {name}[{b},{h}]: {e:.3e}", flush=True)
                    assert np.isfinite(host(got[b, h])).all() and e <= lim, (name, b, h, e, lim)


def test_side_stream_and_caller_buffers():
    """Work is enqueued on the stream handed in (default priority) and lands in the buffers handed
    in; results are bit-identical to the default-stream call."""
    B, H, N, C, R = 2, 2, 500, 128, 8
    q, k, v, dout, pq, pk = _case(B, H, N, C, R, seed=9300)
    d = [dev(x, "bf16") for x in (q, k, v, pq, pk)]
    dd = dev(dout, "bf16")
    o0, l0 = api.fb_lowrank_attn_fwd(*d)
    g0 = api.fb_lowrank_attn_bwd(*d, o0, l0, dd)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    out = torch.full_like(o0, float("nan"))
    lse = torch.full_like(l0, float("nan"))
    grads = tuple(torch.full_like(g, float("nan")) for g in g0)
    ws = torch.empty(api.fb_lowrank_attn_bwd_workspace_bytes(B, H, N, C, R), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    r = api.fb_lowrank_attn_fwd(*d, out=out, lse=lse, stream=side)
    assert r[0] is out and r[1] is lse
    g = api.fb_lowrank_attn_bwd(*d, out, lse, dd, workspace=ws, grads=grads, stream=side)
    side.synchronize()
    assert torch.equal(out, o0) and torch.equal(lse, l0)
    for a, b in zip(g, g0):
        assert torch.equal(a, b)
    for a, b in zip(g, grads):
        assert a is b


def test_binding_rejects_what_it_cannot_pass():
    q = torch.zeros((1, 1, 64, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(api.FlashBiasError):
        api.fb_lowrank_attn_fwd(q.transpose(2, 3), q, q, None, None)          # not contiguous
    with pytest.raises(api.FlashBiasError):
        api.fb_lowrank_attn_fwd(q.cpu(), q, q, None, None)                    # host tensor
    with pytest.raises(api.FlashBiasError):
        api.fb_lowrank_attn_fwd(q.half(), q.half(), q.half(), None, None)     # fp16 has no kernel
    q48 = torch.zeros((1, 1, 64, 48), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(api.FlashBiasError):
        api.fb_lowrank_attn_fwd(q48, q48, q48, None, None)                    # head dimension 48
