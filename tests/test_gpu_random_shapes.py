"""GPU parity over a seeded sweep of valid shapes the hand-picked cases do not list: random
sequence lengths (ragged against every tile size), head dimensions, ranks up to the padded
limit, factor dtypes, masks and batch-shared factors, forward and backward, against the float64
oracle.  The sweep is fixed by its seed; every case prints its shape before it runs."""
import numpy as np
import pytest
import torch

from oracle import fb_oracle as O
from paper_2505_12044_amd import api, workloads as W
from tests._gpu_util import GRAD_TOL, TOL, dev, host, max_abs

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
    assert max_abs(host(out), ro) <= TOL["bf16"] and max_abs(host(lse), rl) <= TOL["bf16"]


@pytest.mark.parametrize("B,H,N,C,R,phi_dtype,causal,shared,seed", _cases(24, 778, True))
def test_backward_random_shape(B, H, N, C, R, phi_dtype, causal, shared, seed):
    print(f"bwd B{B} H{H} N{N} C{C} R{R} {phi_dtype} causal={causal} shared={shared}", flush=True)
    q, k, v, dout, pq, pk = _inputs(B, H, N, C, R, phi_dtype, shared, seed)
    d = [dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), dev(pq, phi_dtype), dev(pk, phi_dtype)]
    out, lse = api.fb_lowrank_attn_fwd(*d, causal=causal)
    grads = api.fb_lowrank_attn_bwd(*d, out, lse, dev(dout, "bf16"), causal=causal)
    torch.cuda.synchronize()
    zero = np.zeros((1, H, N, 0))
    ref = O.batched_attention_lowrank_grads(q, k, v, pq if R else zero, pk if R else zero, dout, causal=causal)
    for name, g, r in zip(("dq", "dk", "dv", "dphi_q", "dphi_k"), grads, ref):
        if g is None:
            continue
        gh = host(g)
        assert np.isfinite(gh).all(), name
        err = max_abs(gh, r) / max(1.0, float(np.abs(r).max()) / 2.5)
        assert err <= GRAD_TOL, (name, err)
