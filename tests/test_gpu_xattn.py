"""GPU parity of the cross-attention entry points (N queries, M keys, N != M; the general
form of Eq. 1) against the float64 oracle, forward and backward."""
import numpy as np
import pytest
import torch

from oracle import fb_oracle as O
from paper_2505_12044_amd import api, workloads as W
from tests._gpu_util import GRAD_TOL, TOL, check_fwd, check_grad, dev, host, max_abs

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
    ro = np.empty((B, H, N, C)); rl = np.empty((B, H, N))
    for b in range(B):
        for h in range(H):
            bias = O.lowrank_bias(pq[b, h], pk[b, h]) if R else None
            ro[b, h], rl[b, h] = O.attention_with_bias(q[b, h], k[b, h], v[b, h], bias)
    label = f"xattn fwd N{N} M{M} C{C} R{R} {phi_dtype}"
    check_fwd(label, "out", host(out), ro)
    check_fwd(label, "lse", host(lse), rl)


# case index -> gradients whose bound scales with the data.  Case 5 has a single key: dv is the sum of
# all 500 rows of dO, entries up to 50, where bf16 storage of the result alone is off by up to 0.12.
DATA_SCALED = {5: ("dv",)}


@pytest.mark.parametrize("idx", range(len(CASES)))
def test_xattn_backward(idx):
    B, H, N, M, C, R, phi_dtype = CASES[idx]
    q, k, v, dout, pq, pk = _problem(B, H, N, M, C, R, phi_dtype, seed=6000 + N + M)
    d = [dev(x, "bf16") for x in (q, k, v)]
    dpq, dpk = dev(pq, phi_dtype), dev(pk, phi_dtype)
    out, lse = api.fb_lowrank_xattn_fwd(*d, dpq, dpk)
    grads = api.fb_lowrank_xattn_bwd(*d, dpq, dpk, out, lse, dev(dout, "bf16"))
    torch.cuda.synchronize()
    for b in range(B):
        for h in range(H):
            if R:
                ref = O.attention_lowrank_grads(q[b, h], k[b, h], v[b, h], pq[b, h], pk[b, h], dout[b, h])
            else:
                ref = O.attention_with_bias_grads(q[b, h], k[b, h], v[b, h], None, dout[b, h])[:3]
            label = f"xattn bwd#{idx} N{N} M{M} C{C} R{R} {phi_dtype} (b,h)=({b},{h})"
            for name, g, r in zip(("dq", "dk", "dv", "dphi_q", "dphi_k"), grads, ref):
                if g is None:
                    continue
                check_grad(label, name, host(g[b, h]), r, data_scaled=name in DATA_SCALED.get(idx, ()))
