"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(automatic kernel choice).  Every (batch, head) pair of all five configurations is touched:
the vision and Pairformer configurations and the low-rank forward of the headline
configuration are compared as whole tensors; elsewhere the oracle computes eight query rows
of every (b, h) one by one (a row of attention is an independent softmax over all keys: the
first and last row of a random query tile, the sequence ends, random rows) plus every row
of some heads.  Gradients: whole tensors for the vision and Pairformer configurations, every
row of three heads for the headline configuration, and for the long-sequence training
configuration the token slice [7777, 8801) — deliberately not tile-aligned — against the
oracle's full-problem chain rule for two (batch, head) pairs.  Every comparison prints the
unscaled max-abs error and the error relative to RMS(ref)."""
import numpy as np
import pytest
import torch

from oracle import fb_oracle as O
from paper_2505_12044_amd import api, workloads as W
from tests._gpu_util import (GRAD_TOL, TOL, check_fwd, check_grad, dev, host, max_abs, oracle_rows_lowrank, report,
                             workload_to_device)

pytestmark = pytest.mark.gpu

# configuration -> gradients whose bound scales with the data (5e-2 * max(1, max|ref| / 2.5)); every
# other gradient of every configuration is held to the flat 5e-2
# (measured: dq, dk, dv of all five configurations, and the factor gradients of the vision,
# long-sequence and PDE configurations, are inside the flat bound at full size).  Pairformer: dphi_q
# reaches 9 and lands at 0.058.  Headline: the slope gradients reach 30 and land at 0.12, 0.4 % of
# the largest entry — the bf16 rounding of q * scale alone moves P, and with it dS, by that much.
FULL_DATA_SCALED = {"pairformer": ("dphi_q", "dphi_k"), "alibi_causal": ("dm_i", "key-side")}


def _sample_rows(N, rng, extra=12):
    fixed = [0, 1, 31, 32, 63, 64, 127, 128, 255, 256, N // 2 - 1, N // 2, N - 129, N - 33, N - 2, N - 1]
    rows = sorted({r for r in fixed if 0 <= r < N} | set(int(x) for x in rng.integers(0, N, extra)))
    return rows


def _few_rows(N, rng, tile=128):
    """Eight rows for an every-(b, h) sweep: the first and last row of a random query tile (the
    kernels remap workgroups to (b, h, tile) units per XCD, so a mapping slip shows as a wrong
    tile), the sequence's first and last row, and random rows."""
    t = int(rng.integers(0, (N + tile - 1) // tile))
    fixed = {0, N - 1, t * tile, min(N - 1, t * tile + tile - 1)}
    while len(fixed) < 8:
        fixed.add(int(rng.integers(0, N)))
    return sorted(fixed)


def _oracle_rows(w, b, h, rows, dense):
    if not dense:
        return oracle_rows_lowrank(w, b, h, rows)
    bb = 0 if w.bias.shape[0] == 1 else b
    ro = np.empty((len(rows), w.C)); rl = np.empty(len(rows))
    for n, r in enumerate(rows):
        o1, l1 = O.attention_with_bias(w.q[b, h, r:r + 1], w.k[b, h], w.v[b, h], w.bias[bb, h, r:r + 1],
                                       causal=w.causal, row_offset=r)
        ro[n], rl[n] = o1[0], l1[0]
    return ro, rl


def _forward(w, d, dense):
    if dense:
        return api.fb_dense_bias_attn_fwd(d["q"], d["k"], d["v"], d["bias"], causal=w.causal)
    return api.fb_lowrank_attn_fwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], causal=w.causal)


def _check_forward_sampled(w, d, dense=False, full_heads=()):
    """Every (b, h): eight sampled rows (tile boundaries + random).  full_heads: (b, h) pairs whose
    whole output is compared, every row."""
    out, lse = _forward(w, d, dense)
    torch.cuda.synchronize()
    rng = np.random.default_rng(7)
    go_all, ro_all, gl_all, rl_all = [], [], [], []
    oh, lh = host(out), host(lse)
    for b in range(w.B):
        for h in range(w.H):
            rows = _few_rows(w.N, rng) if (b, h) not in full_heads else _sample_rows(w.N, rng)
            ro, rl = _oracle_rows(w, b, h, rows, dense)
            go_all.append(oh[b, h, rows]); ro_all.append(ro); gl_all.append(lh[b, h, rows]); rl_all.append(rl)
    kind = "dense" if dense else "lowrank"
    label = f"full-size {kind} {w.name}, sampled rows of all {w.B * w.H} (b,h)"
    check_fwd(label, "out", np.concatenate(go_all), np.concatenate(ro_all), w.dtype)
    check_fwd(label, "lse", np.concatenate(gl_all), np.concatenate(rl_all), w.dtype)
    if full_heads:
        # whole rows of the oracle, a block of 2048 query rows at a time to bound its memory
        go_all, ro_all, gl_all, rl_all = [], [], [], []
        for (b, h) in full_heads:
            bp = 0 if w.phi_q.shape[0] == 1 else b
            for r0 in range(0, w.N, 2048):
                r1 = min(w.N, r0 + 2048)
                if dense:
                    ro, rl = O.attention_with_bias(w.q[b, h, r0:r1], w.k[b, h], w.v[b, h],
                                                   w.bias[0 if w.bias.shape[0] == 1 else b, h, r0:r1],
                                                   causal=w.causal, row_offset=r0)
                else:
                    ro, rl = O.attention_lowrank(w.q[b, h, r0:r1], w.k[b, h], w.v[b, h], w.phi_q[bp, h, r0:r1],
                                                 w.phi_k[bp, h], causal=w.causal, row_offset=r0)
                go_all.append(oh[b, h, r0:r1]); ro_all.append(ro); gl_all.append(lh[b, h, r0:r1]); rl_all.append(rl)
        label = f"full-size {kind} {w.name}, every row of {len(full_heads)} (b,h)"
        check_fwd(label, "out", np.concatenate(go_all), np.concatenate(ro_all), w.dtype)
        check_fwd(label, "lse", np.concatenate(gl_all), np.concatenate(rl_all), w.dtype)
    return out, lse


def _check_forward_whole(w, d, dense=False):
    """The whole output tensor, every (b, h) and row."""
    out, lse = _forward(w, d, dense)
    torch.cuda.synchronize()
    if dense:
        ro, rl = O.batched_attention_dense(w.q, w.k, w.v, w.bias, causal=w.causal)
    else:
        ro, rl = O.batched_attention_lowrank(w.q, w.k, w.v, w.phi_q, w.phi_k, causal=w.causal)
    label = f"full-size {'dense' if dense else 'lowrank'} {w.name}, whole tensor"
    check_fwd(label, "out", host(out), ro, w.dtype)
    check_fwd(label, "lse", host(lse), rl, w.dtype)
    return out, lse


def _check_backward_whole(w, d, out, lse, data_scaled=()):
    """Whole-tensor gradients of a configuration with batch-shared factors (per-batch dphi).  Flat
    5e-2 unless a gradient is named in data_scaled."""
    grads = api.fb_lowrank_attn_bwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], out, lse, d["dout"],
                                    causal=w.causal)
    torch.cuda.synchronize()
    ref = O.batched_attention_lowrank_grads(w.q, w.k, w.v, w.phi_q, w.phi_k, w.dout, causal=w.causal)
    label = f"full-size backward {w.name}, whole tensor"
    for name, g, r in zip(("dq", "dk", "dv", "dphi_q", "dphi_k"), grads, ref):
        check_grad(label, name, host(g), r, data_scaled=name in data_scaled)


def test_alibi_causal_full():
    """Headline configuration.  Low-rank kernel: the whole output, every row of all 64 (b, h).
    Dense kernel: eight rows of every (b, h) and every row of eight heads."""
    w = W.make_workload("alibi_causal", dense=True)
    d = workload_to_device(w, dense=True)
    _check_forward_sampled(w, d, full_heads=[(b, h) for b in range(w.B) for h in range(w.H)])
    _check_forward_sampled(w, d, dense=True, full_heads=[(b, (5 * b + 2 * i) % w.H) for b in range(w.B) for i in range(2)])


def test_vision_relpos_full():
    """Whole tensor, low-rank and dense forward, and the whole backward."""
    w = W.make_workload("vision_relpos", dense=True, with_dout=True)
    d = workload_to_device(w, dense=True)
    out, lse = _check_forward_whole(w, d)
    o2, _ = _check_forward_whole(w, d, dense=True)
    # the rank-32 factors approximate the dense table: report, and bound loosely, the
    # end-to-end deviation between the two kernels' outputs (an approximation error, not a
    # kernel error)
    dev_max = float((out.float() - o2.float()).abs().max())
    energy = min(O.svd_energy(w.bias_exact[0, h], 32) for h in range(w.H))
    print(f"vision_relpos: rank-32 energy >= {energy:.5f}; lowrank-vs-dense output deviation {dev_max:.3e}", flush=True)
    assert energy > 0.99 and dev_max < 0.15
    _check_backward_whole(w, d, out, lse, data_scaled=FULL_DATA_SCALED.get("vision_relpos", ()))


def test_pairformer_full():
    """Whole tensor (all 1536 (b, h)), low-rank and dense forward, and the whole backward."""
    w = W.make_workload("pairformer", dense=True, with_dout=True)
    d = workload_to_device(w, dense=True)
    out, lse = _check_forward_whole(w, d)
    _check_forward_whole(w, d, dense=True)
    _check_backward_whole(w, d, out, lse, data_scaled=FULL_DATA_SCALED.get("pairformer", ()))


def test_long_train_full_forward_and_gradients():
    """Eight rows of every (b, h) and every row of one head; gradients on the unaligned token slice
    [7777, 8801) of two heads at the flat 5e-2."""
    w = W.make_workload("long_train")
    d = workload_to_device(w)
    out, lse = _check_forward_sampled(w, d, full_heads=[(1, 5)])
    grads = api.fb_lowrank_attn_bwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], out, lse, d["dout"])
    torch.cuda.synchronize()
    lo, hi = 7777, 8801
    names = ("dq", "dk", "dv", "dphi_q", "dphi_k")
    for (b, h) in [(0, 0), (1, 7)]:
        ref = O.attention_lowrank_grads(w.q[b, h], w.k[b, h], w.v[b, h], w.phi_q[b, h], w.phi_k[b, h],
                                        w.dout[b, h], row_block=1024)
        label = f"long_train gradients, slice [{lo},{hi}) of (b,h)=({b},{h})"
        for name, g, r in zip(names, grads, ref):
            check_grad(label, name, host(g[b, h, lo:hi]), r[lo:hi])


def test_pde_distance_full_forward_and_gradients():
    """The PDE-solver shape (Sec. 4.3): N = 32186 (no multiple of any tile), C = 16, rank-9 fp32
    distance factors.  Forward rows against the oracle on bias rows materialised from the
    definition -s alpha_i ||x_i - x_j||^2; gradients of one head on an unaligned token slice
    against the oracle's chain rule (bound scaled with the data as for the small cases)."""
    w = W.make_pde_workload()
    x, alpha, s = w.notes["x"], w.notes["alpha"], w.notes["strength"]
    d = workload_to_device(w)
    out, lse = api.fb_lowrank_attn_fwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"])
    grads = api.fb_lowrank_attn_bwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], out, lse, d["dout"])
    torch.cuda.synchronize()
    rng = np.random.default_rng(11)
    go_all, ro_all, gl_all, rl_all = [], [], [], []
    for h in range(w.H):
        rows = _sample_rows(w.N, rng) if h in (0, 5, 7) else _few_rows(w.N, rng)
        go_all.append(host(out[0, h, rows])); gl_all.append(host(lse[0, h, rows]))
        for r in rows:
            brow = -s * alpha[h, r] * O.squared_distance_bias(x[r:r + 1], x)
            o1, l1 = O.attention_with_bias(w.q[0, h, r:r + 1], w.k[0, h], w.v[0, h], brow, row_offset=r)
            ro_all.append(o1); rl_all.append(l1)
    check_fwd("full-size pde_distance, sampled rows of every head", "out", np.concatenate(go_all), np.concatenate(ro_all))
    check_fwd("full-size pde_distance, sampled rows of every head", "lse", np.concatenate(gl_all), np.concatenate(rl_all))
    h, lo, hi = 3, 15001, 16025
    ref = O.attention_lowrank_grads(w.q[0, h], w.k[0, h], w.v[0, h], w.phi_q[0, h], w.phi_k[0, h],
                                    w.dout[0, h], row_block=512)
    label = f"pde_distance gradients, slice [{lo},{hi}) of head {h}"
    for name, g, r in zip(("dq", "dk", "dv", "dphi_q", "dphi_k"), grads, ref):
        check_grad(label, name, host(g[0, h, lo:hi]), r[lo:hi], data_scaled=name in FULL_DATA_SCALED.get("pde_distance", ()))


def test_alibi_causal_full_gradients():
    """The headline shape's backward (causal tile pairs, fp32 rank-2 ALiBi factors) at full size:
    every gradient row of three heads (steepest, middle and flattest slope) against the oracle.
    dq, dk, dv: 5e-2, scaled with the data where the reference exceeds 2.5.
    The raw factor gradients are ill-conditioned at this length: rows of dS sum to zero in exact
    arithmetic, and sum_j dS_ij * j with absolute positions j <= N multiplies any violation of
    that (D = rowsum(dO o O) is taken from the bf16 output, 2^-9 relative) by N.  What a model
    can use is the chain rule onto the slope, phi_q(i) = [-m i, m] -> dm_i = dphi_q[i,1] -
    i dphi_q[i,0] = sum_j dS_ij (j - i), and its key-side mirror dphi_k[j,0] + j dphi_k[j,1] =
    -m sum_i dS_ij (i - j); these are checked, to the same bound."""
    w = W.make_workload("alibi_causal", with_dout=True)
    d = workload_to_device(w)
    out, lse = api.fb_lowrank_attn_fwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], causal=True)
    grads = api.fb_lowrank_attn_bwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], out, lse, d["dout"], causal=True)
    torch.cuda.synchronize()
    pos = np.arange(w.N, dtype=np.float64)
    for (b, h) in [(0, 0), (2, 7), (3, 15)]:
        ref = O.attention_lowrank_grads(w.q[b, h], w.k[b, h], w.v[b, h], w.phi_q[0, h], w.phi_k[0, h],
                                        w.dout[b, h], causal=True, row_block=1024)
        label = f"alibi_causal gradients, every row of (b,h)=({b},{h})"
        scaled = FULL_DATA_SCALED.get("alibi_causal", ())
        for name, g, r in zip(("dq", "dk", "dv"), grads, ref):
            check_grad(label, name, host(g[b, h]), r, data_scaled=name in scaled)
        gq, gk = host(grads[3][b, h]), host(grads[4][b, h])
        assert np.isfinite(gq).all() and np.isfinite(gk).all()
        for name, gc, rc in (("dm_i", gq[:, 1] - pos * gq[:, 0], ref[3][:, 1] - pos * ref[3][:, 0]),
                             ("key-side", gk[:, 0] + pos * gk[:, 1], ref[4][:, 0] + pos * ref[4][:, 1])):
            check_grad(label, name, gc, rc, data_scaled=name in scaled)
        # the raw factor gradients, reported (not gated: ill-conditioned at this length, see the docstring)
        for name, g, r in (("dphi_q (raw, reported only)", gq, ref[3]), ("dphi_k (raw, reported only)", gk, ref[4])):
            report(label, name, g, r)
