"""GPU parity on inputs that drive the online softmax through its rare paths (Corollary 3.7's
tiled evaluation keeps a running row maximum and sum): a bias that rises along the keys so that
the running reference is replaced in every block, a single outlier key far into the sequence
(the reference chosen in the first blocks is off by e^60), a large negative constant on every
score, and the same under the causal mask — in every forward kernel variant and in the dense
baseline.  The biases are exact rank-1/rank-2 fp32 factors, so the oracle's dense bias and the
kernel's factor product agree to fp32 rounding."""
import numpy as np
import pytest
import torch

from oracle import fb_oracle as O
from paper_2505_12044_amd import api, workloads as W
from tests._gpu_util import TOL, dev, host, max_abs

pytestmark = pytest.mark.gpu

N, C, H = 700, 64, 2


def _qkv(seed):
    rng = np.random.default_rng(seed)
    return [W.round_bf16(rng.standard_normal((1, H, N, C)).astype(np.float32)) for _ in range(3)]


def _factors(kind):
    j = np.arange(N, dtype=np.float32)
    one = np.ones(N, dtype=np.float32)
    if kind == "rising":          # b_ij = 0.5 j : the row maximum moves with every key
        pq, pk = one[:, None], (0.5 * j)[:, None]
    elif kind == "outlier":       # b_ij = 60 at key 517 (and 40 at key 3 so that early blocks set a reference)
        col = np.zeros(N, dtype=np.float32); col[517] = 60.0; col[3] = 40.0
        pq, pk = one[:, None], col[:, None]
    elif kind == "shifted":       # b_ij = -3000 - 0.01 i : a huge row-constant shift
        pq = np.stack([-3000.0 * one, -0.01 * j], axis=1)
        pk = np.stack([one, one], axis=1)
    elif kind == "falling":       # b_ij = -0.7 |..| style recency ramp, walked against the causal order
        pq, pk = one[:, None], (-0.7 * j)[:, None]
    pq = np.broadcast_to(pq.astype(np.float32), (1, H) + pq.shape).copy()
    pk = np.broadcast_to(pk.astype(np.float32), (1, H) + pk.shape).copy()
    return pq, pk


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("kind", ["rising", "outlier", "shifted", "falling"])
def test_reference_replacement_paths(kind, causal):
    q, k, v = _qkv(seed=9500)
    pq, pk = _factors(kind)
    d = [dev(x, "bf16") for x in (q, k, v)] + [dev(pq, "f32"), dev(pk, "f32")]
    ref = []
    for h in range(H):
        bias = O.lowrank_bias(pq[0, h], pk[0, h])
        ref.append(O.attention_with_bias(q[0, h], k[0, h], v[0, h], bias, causal=causal))
    worst = 0.0
    for qb in (1, 2, 8, 16):
        api.fb_tune_set("fwd_qb", qb)
        try:
            out, lse = api.fb_lowrank_attn_fwd(*d, causal=causal)
            torch.cuda.synchronize()
        finally:
            api.fb_tune_set("fwd_qb", 0)
        go, gl = host(out), host(lse)
        assert np.isfinite(go).all() and np.isfinite(gl).all(), (kind, qb)
        for h in range(H):
            eo, el = max_abs(go[0, h], ref[h][0]), max_abs(gl[0, h], ref[h][1])
            # lse carries the bias magnitude (up to 3000): fp32 output rounding is 2^-24 relative
            tol_l = TOL["bf16"] + 2.0 ** -22 * float(np.abs(ref[h][1]).max())
            assert eo <= TOL["bf16"] and el <= tol_l, (kind, causal, qb, eo, el)
            worst = max(worst, eo)
    # dense baseline on the same bias (bf16 storage of the bias: compare against the oracle on the rounded bias)
    bias = np.stack([W.round_bf16(O.lowrank_bias(pq[0, h], pk[0, h]).astype(np.float32)) for h in range(H)])[None]
    out, lse = api.fb_dense_bias_attn_fwd(d[0], d[1], d[2], dev(bias, "bf16"), causal=causal)
    torch.cuda.synchronize()
    for h in range(H):
        ro, rl = O.attention_with_bias(q[0, h], k[0, h], v[0, h], bias[0, h], causal=causal)
        assert max_abs(host(out[0, h]), ro) <= TOL["bf16"]
        assert max_abs(host(lse[0, h]), rl) <= TOL["bf16"] + 2.0 ** -22 * float(np.abs(rl).max())
    print(f"softmax paths {kind} causal={causal}: worst out err {worst:.3e}", flush=True)
