"""GPU parity on the paper's second exact decomposition: the squared 3-D distance bias with a
token-wise weight, b_ij = -s alpha_i ||x_i - x_j||^2 (Example 3.5 and the learnable alpha of
the PDE-solver experiment, Sec. 4.3), supplied as the rank-9 factors in fp32.  The sequence
length is ragged (not a multiple of any tile).  The reference is the oracle run on the dense
bias materialised from the definition, so the test also covers the factorisation itself.
The backward check follows the paper's training recipe: the gradient of alpha is obtained from
the factor gradient, d alpha_i = sum_r dphi_q[i, r] * d phi_q[i, r] / d alpha_i, and compared
with the oracle's dense-bias gradient contracted with ||x_i - x_j||^2."""
import numpy as np
import pytest
import torch

from oracle import fb_oracle as O
from paper_2505_12044_amd import api, workloads as W
from tests._gpu_util import GRAD_TOL, TOL, check_fwd, check_grad, dev, host, max_abs

pytestmark = pytest.mark.gpu

S = 4.0   # bias strength: distances in the unit cube are at most 3


def _problem(N, C, H, seed):
    rng = np.random.default_rng(seed)
    q, k, v, dout = (W.round_bf16(rng.standard_normal((1, H, N, C)).astype(np.float32)) for _ in range(4))
    x = rng.random((N, 3))
    alpha = 0.5 + rng.random(N)
    uq, uk = O.squared_distance_factors(x, x)              # float64, unscaled
    phi_q = (-S * alpha[:, None] * uq).astype(np.float32)
    phi_k = uk.astype(np.float32)
    phi_q = np.broadcast_to(phi_q, (1, H, N, 9)).copy()
    phi_k = np.broadcast_to(phi_k, (1, H, N, 9)).copy()
    dist2 = O.squared_distance_bias(x, x)
    bias = -S * alpha[:, None] * dist2
    return q, k, v, dout, phi_q, phi_k, uq, dist2, bias


DATA_SCALED = {}     # (N, C) -> gradients whose bound scales with the data


@pytest.mark.parametrize("N,C", [(1500, 32), (777, 64), (520, 128), (2100, 16)])
def test_distance_bias_forward_and_alpha_gradient(N, C):
    H = 2
    q, k, v, dout, phi_q, phi_k, uq, dist2, bias = _problem(N, C, H, seed=5000 + N)
    dq_, dk_, dv_ = dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16")
    pq, pk = dev(phi_q, "f32"), dev(phi_k, "f32")
    out, lse = api.fb_lowrank_attn_fwd(dq_, dk_, dv_, pq, pk)
    grads = api.fb_lowrank_attn_bwd(dq_, dk_, dv_, pq, pk, out, lse, dev(dout, "bf16"))
    torch.cuda.synchronize()
    for h in range(H):
        label = f"distance bias N{N} C{C} head {h}"
        ro, rl = O.attention_with_bias(q[0, h], k[0, h], v[0, h], bias)
        check_fwd(label, "out", host(out[0, h]), ro)
        check_fwd(label, "lse", host(lse[0, h]), rl)
        rdq, rdk, rdv, rdb = O.attention_with_bias_grads(q[0, h], k[0, h], v[0, h], bias, dout[0, h])
        for name, g, r in (("dq", grads[0], rdq), ("dk", grads[1], rdk), ("dv", grads[2], rdv)):
            check_grad(label, name, host(g[0, h]), r, data_scaled=name in DATA_SCALED.get((N, C), ()))
        dalpha_ref = np.sum(rdb * (-S * dist2), axis=1)
        dalpha_gpu = np.sum(host(grads[3][0, h]) * (-S * uq), axis=1)
        # d alpha sums nine factor gradients weighted by |factor| up to 2 S: bound relative to its size
        check_grad(label, "dalpha", dalpha_gpu, dalpha_ref, gain=max(1.0, float(np.abs(dalpha_ref).max())))


RANK5_DATA_SCALED = ()


def test_distance_bias_rank5_factors():
    """The merged rank-5 form of the same bias (|x|^2 + |y|^2 - 2 x.y): 30 limb columns, padded
    width 32 instead of 64.  Forward and gradients against the oracle on the dense bias."""
    w = W.make_pde_workload(N=1100, H=2, rank5=True)
    x, alpha, s = w.notes["x"], w.notes["alpha"], w.notes["strength"]
    d = [dev(a, "bf16") for a in (w.q, w.k, w.v)] + [dev(w.phi_q, "f32"), dev(w.phi_k, "f32")]
    out, lse = api.fb_lowrank_attn_fwd(*d)
    grads = api.fb_lowrank_attn_bwd(*d, out, lse, dev(w.dout, "bf16"))
    torch.cuda.synchronize()
    for h in range(2):
        bias = -s * alpha[h][:, None] * O.squared_distance_bias(x, x)
        label = f"distance bias rank 5, head {h}"
        ro, rl = O.attention_with_bias(w.q[0, h], w.k[0, h], w.v[0, h], bias)
        check_fwd(label, "out", host(out[0, h]), ro)
        check_fwd(label, "lse", host(lse[0, h]), rl)
        rdq, rdk, rdv, _ = O.attention_with_bias_grads(w.q[0, h], w.k[0, h], w.v[0, h], bias, w.dout[0, h])
        for name, g, r in (("dq", grads[0], rdq), ("dk", grads[1], rdk), ("dv", grads[2], rdv)):
            check_grad(label, name, host(g[0, h]), r, data_scaled=name in RANK5_DATA_SCALED)
