"""GPU parity of the cross-attention entry points (N queries, M keys, N != M; the general
form of Eq. 1) against the float64 oracle, forward and backward."""
import numpy as np
import pytest
import torch

from oracle import fb_oracle as O
from paper_2505_12044_amd import api, workloads as W
from tests._gpu_util import GRAD_TOL, TOL, dev, host, max_abs

pytestmark = pytest.mark.gpu


def _problem(B, H, N, M, C, R, phi_dtype, seed):
    rng = np.random.default_rng(seed)
    rd = lambda shape: W.round_bf16(rng.standard_normal(shape).astype(np.float32))
    q, dout = rd((B, H, N, C)), rd((B, H, N, C))
    k, v = rd((B, H, M, C)), rd((B, H, M, C))
    if R:
        sc = R ** -0.25
        pq = (sc * rng.standard_normal((B, H, N, R))).astype(np.float32)
        pk = (sc * rng.standard_normal((B, H, M, R))).astype(np.float32)
        if phi_dtype == "bf16":
            pq, pk = W.round_bf16(pq), W.round_bf16(pk)
    else:
        pq = pk = None
    return q, k, v, dout, pq, pk


CASES = [(2, 2, 300, 1000, 128, 8, "bf16"), (1, 3, 1000, 300, 64, 16, "bf16"), (2, 2, 129, 33, 32, 3, "f32"),
         (1, 2, 64, 4096, 128, 0, "bf16"), (1, 1, 1, 77, 64, 5, "bf16"), (1, 2, 500, 1, 128, 8, "bf16"),
         (2, 2, 300, 1001, 16, 8, "bf16"), (1, 2, 131, 333, 16, 9, "f32")]


@pytest.mark.parametrize("B,H,N,M,C,R,phi_dtype", CASES)
def test_xattn_forward(B, H, N, M, C, R, phi_dtype):
    q, k, v, dout, pq, pk = _problem(B, H, N, M, C, R, phi_dtype, seed=6000 + N + M)
    out, lse = api.fb_lowrank_xattn_fwd(dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"),
                                        dev(pq, phi_dtype), dev(pk, phi_dtype))
    torch.cuda.synchronize()
    eo = el = 0.0
    for b in range(B):
        for h in range(H):
            bias = O.lowrank_bias(pq[b, h], pk[b, h]) if R else None
            ro, rl = O.attention_with_bias(q[b, h], k[b, h], v[b, h], bias)
            eo = max(eo, max_abs(host(out[b, h]), ro))
            el = max(el, max_abs(host(lse[b, h]), rl))
    print(f"xattn fwd N{N} M{M} C{C} R{R} {phi_dtype}: out {eo:.3e} lse {el:.3e}", flush=True)
    assert eo <= TOL["bf16"] and el <= TOL["bf16"]


@pytest.mark.parametrize("B,H,N,M,C,R,phi_dtype", CASES)
def test_xattn_backward(B, H, N, M, C, R, phi_dtype):
    q, k, v, dout, pq, pk = _problem(B, H, N, M, C, R, phi_dtype, seed=6000 + N + M)
    d = [dev(x, "bf16") for x in (q, k, v)]
    dpq, dpk = dev(pq, phi_dtype), dev(pk, phi_dtype)
    out, lse = api.fb_lowrank_xattn_fwd(*d, dpq, dpk)
    grads = api.fb_lowrank_xattn_bwd(*d, dpq, dpk, out, lse, dev(dout, "bf16"))
    torch.cuda.synchronize()
    worst = 0.0
    for b in range(B):
        for h in range(H):
            if R:
                ref = O.attention_lowrank_grads(q[b, h], k[b, h], v[b, h], pq[b, h], pk[b, h], dout[b, h])
            else:
                ref = O.attention_with_bias_grads(q[b, h], k[b, h], v[b, h], None, dout[b, h])[:3]
            for g, r in zip(grads, ref):
                if g is None:
                    continue
                gh = host(g[b, h])
                assert np.isfinite(gh).all()
                worst = max(worst, max_abs(gh, r) / max(1.0, float(np.abs(r).max()) / 2.5))
    print(f"xattn bwd N{N} M{M} C{C} R{R} {phi_dtype}: worst scaled err {worst:.3e}", flush=True)
    assert worst <= GRAD_TOL
