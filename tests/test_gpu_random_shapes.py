"""GPU parity over a seeded sweep of valid shapes the hand-picked cases do not list: random
sequence lengths (ragged against every tile size), head dimensions, ranks up to the padded
limit, factor dtypes, masks and batch-shared factors, forward and backward, against the float64
oracle.  The sweep is fixed by its seed; every case prints its shape before it runs."""
import numpy as np
import pytest
import torch

from oracle import fb_oracle as O
from paper_2505_12044_amd import api, workloads as W
from tests._gpu_util import GRAD_TOL, TOL, check_fwd, check_grad, dev, host, max_abs

pytestmark = pytest.mark.gpu


def _cases(n, seed, backward):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        C = int(rng.choice([16, 32, 64, 128]))
        f32 = bool(rng.integers(0, 2))
        R = int(rng.integers(0, 11)) if f32 else int(rng.integers(0, 65))
        N = int(rng.choice([rng.integers(1, 64), rng.integers(64, 300), rng.integers(300, 700)]))
        B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
        causal = bool(rng.integers(0, 2))
        shared = bool(rng.integers(0, 2))
        out.append((B, H, N, C, R, "f32" if f32 else "bf16", causal, shared, int(rng.integers(1 << 30))))
    return out


def _factor_gain(name, pq, pk):
    """The backward takes D_i = sum_c dout * out from the bf16 `out` it is handed, so dS carries
    an error P_ij * dD_i; in dq and dk that meets k * scale and q * scale (below 1 in magnitude),
    in dphi_q = dS phi_k and dphi_k = dS^T phi_q it meets the other side's factors unscaled.  The
    gradient bar, stated for O(1) operands, therefore scales with max |phi| of the other side
    (rank-1 fp32 factors of this sweep reach 4)."""
    if name == "dphi_q":
        return max(1.0, float(np.abs(pk).max()))
    if name == "dphi_k":
        return max(1.0, float(np.abs(pq).max()))
    return 1.0


def _inputs(B, H, N, C, R, phi_dtype, shared, seed):
    rng = np.random.default_rng(seed)
    rd = lambda *s: W.round_bf16(rng.standard_normal(s).astype(np.float32))
    q, k, v, dout = rd(B, H, N, C), rd(B, H, N, C), rd(B, H, N, C), rd(B, H, N, C)
    Bp = 1 if shared else B
    pq = pk = None
    if R:
        sc = R ** -0.25
        pq = (sc * rng.standard_normal((Bp, H, N, R))).astype(np.float32)
        pk = (sc * rng.standard_normal((Bp, H, N, R))).astype(np.float32)
        if phi_dtype == "bf16":
            pq, pk = W.round_bf16(pq), W.round_bf16(pk)
    return q, k, v, dout, pq, pk


@pytest.mark.parametrize("B,H,N,C,R,phi_dtype,causal,shared,seed", _cases(40, 777, False))
def test_forward_random_shape(B, H, N, C, R, phi_dtype, causal, shared, seed):
    print(f"fwd B{B} H{H} N{N} C{C} R{R} {phi_dtype} causal={causal} shared={shared}", flush=True)
    q, k, v, _, pq, pk = _inputs(B, H, N, C, R, phi_dtype, shared, seed)
    out, lse = api.fb_lowrank_attn_fwd(dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"),
                                       dev(pq, phi_dtype), dev(pk, phi_dtype), causal=causal)
    torch.cuda.synchronize()
    ro, rl = O.batched_attention_lowrank(q, k, v, pq if R else np.zeros((1, H, N, 0)),
                                         pk if R else np.zeros((1, H, N, 0)), causal=causal)
    label = f"fwd B{B} H{H} N{N} C{C} R{R} {phi_dtype} causal={causal} shared={shared}"
    check_fwd(label, "out", host(out), ro)
    check_fwd(label, "lse", host(lse), rl)


BWD_CASES = _cases(24, 778, True)
# sweep index -> gradients of that case whose bound scales with the data (entries of magnitude 10+)
BWD_DATA_SCALED = {}


@pytest.mark.parametrize("idx", range(len(BWD_CASES)))
def test_backward_random_shape(idx):
    B, H, N, C, R, phi_dtype, causal, shared, seed = BWD_CASES[idx]
    print(f"bwd B{B} H{H} N{N} C{C} R{R} {phi_dtype} causal={causal} shared={shared}", flush=True)
    q, k, v, dout, pq, pk = _inputs(B, H, N, C, R, phi_dtype, shared, seed)
    d = [dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), dev(pq, phi_dtype), dev(pk, phi_dtype)]
    out, lse = api.fb_lowrank_attn_fwd(*d, causal=causal)
    grads = api.fb_lowrank_attn_bwd(*d, out, lse, dev(dout, "bf16"), causal=causal)
    torch.cuda.synchronize()
    zero = np.zeros((1, H, N, 0))
    ref = O.batched_attention_lowrank_grads(q, k, v, pq if R else zero, pk if R else zero, dout, causal=causal)
    label = f"bwd#{idx} B{B} H{H} N{N} C{C} R{R} {phi_dtype} causal={causal} shared={shared}"
    for name, g, r in zip(("dq", "dk", "dv", "dphi_q", "dphi_k"), grads, ref):
        if g is None:
            continue
        check_grad(label, name, host(g), r, data_scaled=name in BWD_DATA_SCALED.get(idx, ()),
                   gain=_factor_gain(name, pq, pk))


def _xcases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        C = int(rng.choice([16, 32, 64, 128]))
        f32 = bool(rng.integers(0, 2))
        R = int(rng.integers(0, 11)) if f32 else int(rng.integers(0, 65))
        N, M = int(rng.integers(1, 500)), int(rng.integers(1, 900))
        out.append((int(rng.integers(1, 3)), int(rng.integers(1, 3)), N, M, C, R, "f32" if f32 else "bf16",
                    int(rng.integers(1 << 30))))
    return out


X_CASES = _xcases(16, 779)
X_DATA_SCALED = {}


@pytest.mark.parametrize("idx", range(len(X_CASES)))
def test_xattn_random_shape(idx):
    B, H, N, M, C, R, phi_dtype, seed = X_CASES[idx]
    print(f"xattn B{B} H{H} N{N} M{M} C{C} R{R} {phi_dtype}", flush=True)
    rng = np.random.default_rng(seed)
    rd = lambda *s: W.round_bf16(rng.standard_normal(s).astype(np.float32))
    q, dout, k, v = rd(B, H, N, C), rd(B, H, N, C), rd(B, H, M, C), rd(B, H, M, C)
    pq = pk = None
    if R:
        pq = (R ** -0.25 * rng.standard_normal((B, H, N, R))).astype(np.float32)
        pk = (R ** -0.25 * rng.standard_normal((B, H, M, R))).astype(np.float32)
        if phi_dtype == "bf16":
            pq, pk = W.round_bf16(pq), W.round_bf16(pk)
    d = [dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), dev(pq, phi_dtype), dev(pk, phi_dtype)]
    out, lse = api.fb_lowrank_xattn_fwd(*d)
    grads = api.fb_lowrank_xattn_bwd(*d, out, lse, dev(dout, "bf16"))
    torch.cuda.synchronize()
    for b in range(B):
        for h in range(H):
            fq = pq[b, h] if R else np.zeros((N, 0))
            fk = pk[b, h] if R else np.zeros((M, 0))
            ro, rl = O.attention_lowrank(q[b, h], k[b, h], v[b, h], fq, fk)
            label = f"xattn#{idx} N{N} M{M} C{C} R{R} {phi_dtype} (b,h)=({b},{h})"
            check_fwd(label, "out", host(out[b, h]), ro)
            check_fwd(label, "lse", host(lse[b, h]), rl)
            ref = O.attention_lowrank_grads(q[b, h], k[b, h], v[b, h], fq, fk, dout[b, h])
            for name, g, r in zip(("dq", "dk", "dv", "dphi_q", "dphi_k"), grads, ref):
                if g is None:
                    continue
                check_grad(label, name, host(g[b, h]), r, data_scaled=name in X_DATA_SCALED.get(idx, ()),
                           gain=_factor_gain(name, pq, pk))


def _dcases(n, seed):
    rng = np.random.default_rng(seed)
    return [(int(rng.integers(1, 3)), int(rng.integers(1, 3)), 8 * int(rng.integers(1, 70)),
             int(rng.choice([16, 32, 64, 128])), bool(rng.integers(0, 2)), bool(rng.integers(0, 2)),
             int(rng.integers(1 << 30))) for _ in range(n)]


D_CASES = _dcases(12, 780)
D_DATA_SCALED = {}


@pytest.mark.parametrize("idx", range(len(D_CASES)))
def test_dense_random_shape(idx):
    B, H, N, C, causal, shared, seed = D_CASES[idx]
    print(f"dense B{B} H{H} N{N} C{C} causal={causal} shared={shared}", flush=True)
    rng = np.random.default_rng(seed)
    rd = lambda *s: W.round_bf16(rng.standard_normal(s).astype(np.float32))
    q, k, v, dout = rd(B, H, N, C), rd(B, H, N, C), rd(B, H, N, C), rd(B, H, N, C)
    bias = rd(1 if shared else B, H, N, N)
    d = [dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), dev(bias, "bf16")]
    out, lse = api.fb_dense_bias_attn_fwd(*d, causal=causal)
    grads = api.fb_dense_bias_attn_bwd(*d, out, lse, dev(dout, "bf16"), causal=causal)
    torch.cuda.synchronize()
    for b in range(B):
        for h in range(H):
            bb = bias[0 if shared else b, h]
            ro, rl = O.attention_with_bias(q[b, h], k[b, h], v[b, h], bb, causal=causal)
            label = f"dense#{idx} N{N} C{C} causal={causal} shared={shared} (b,h)=({b},{h})"
            check_fwd(label, "out", host(out[b, h]), ro)
            check_fwd(label, "lse", host(lse[b, h]), rl)
            ref = O.attention_with_bias_grads(q[b, h], k[b, h], v[b, h], bb, dout[b, h], causal=causal)
            for name, g, r in zip(("dq", "dk", "dv", "dbias"), grads, ref):
                if name == "dbias" and causal:
                    r = np.tril(r)
                check_grad(label, name, host(g[b, h]), r, data_scaled=name in D_DATA_SCALED.get(idx, ()))
