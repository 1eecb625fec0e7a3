"""GPU parity: HIP forward kernels (through the C-ABI binding) against the float64 oracle,
element by element on the same seeded inputs.  Tolerances: max abs error 1e-4 (fp32),
2e-2 (bf16) on out and lse."""
import numpy as np
import pytest
import torch

from oracle import fb_oracle as O
from paper_2505_12044_amd import api, workloads as W
from tests._gpu_util import TOL, dev, host, max_abs, oracle_rows_lowrank, workload_to_device

pytestmark = pytest.mark.gpu


def _check_lowrank(w, qb=0):
    d = workload_to_device(w)
    api.fb_tune_set("fwd_qb", qb)
    try:
        out, lse = api.fb_lowrank_attn_fwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], causal=w.causal)
        torch.cuda.synchronize()
    finally:
        api.fb_tune_set("fwd_qb", 0)
    ro, rl = O.batched_attention_lowrank(w.q, w.k, w.v, w.phi_q, w.phi_k, causal=w.causal)
    eo, el = max_abs(host(out), ro), max_abs(host(lse), rl)
    print(f"{w.name} B{w.B} H{w.H} N{w.N} C{w.C} R{w.R} qb={qb}: out err {eo:.3e}, lse err {el:.3e}", flush=True)
    assert np.isfinite(host(out)).all() and np.isfinite(host(lse)).all()
    assert eo <= TOL[w.dtype] and el <= TOL[w.dtype]
    return out, lse


def _check_dense(w, qb=0):
    d = workload_to_device(w, dense=True)
    api.fb_tune_set("fwd_qb", qb)
    try:
        out, lse = api.fb_dense_bias_attn_fwd(d["q"], d["k"], d["v"], d["bias"], causal=w.causal)
        torch.cuda.synchronize()
    finally:
        api.fb_tune_set("fwd_qb", 0)
    ro, rl = O.batched_attention_dense(w.q, w.k, w.v, w.bias, causal=w.causal)
    eo, el = max_abs(host(out), ro), max_abs(host(lse), rl)
    print(f"dense {w.name} B{w.B} H{w.H} N{w.N} C{w.C} qb={qb}: out err {eo:.3e}, lse err {el:.3e}", flush=True)
    assert eo <= TOL[w.dtype] and el <= TOL[w.dtype]


def test_config1_tiny_fp32_full():
    w = W.make_workload("tiny_fp32", dense=True)
    _check_lowrank(w)
    _check_dense(w)


@pytest.mark.parametrize("N,C,R,causal", [(200, 32, 3, True), (77, 128, 9, False), (129, 64, 0, True), (150, 16, 4, False)])
def test_fp32_ragged(N, C, R, causal):
    w = W.make_workload("tiny_fp32", dense=True, B=2, H=2, N=N, C=C, R=R, causal=causal)
    _check_lowrank(w)
    _check_dense(w)


SMALL = [
    ("alibi_causal", dict(B=2, H=4, N=512)),
    ("alibi_causal", dict(B=1, H=2, N=333)),            # ragged tail, causal, fp32 factors
    ("vision_relpos", dict(B=2, H=3, N=256)),
    ("pairformer", dict(B=5, N=384)),
    ("long_train", dict(B=1, H=2, N=1024)),
    ("long_train", dict(B=1, H=1, N=1000, R=5)),        # ragged, bf16 factors with R % 8 != 0
]


@pytest.mark.parametrize("qb", [1, 2, 8, 16])
@pytest.mark.parametrize("name,ov", SMALL)
def test_bf16_lowrank_small(name, ov, qb):
    _check_lowrank(W.make_workload(name, **ov), qb=qb)


@pytest.mark.parametrize("qb", [1, 2, 8, 16])
@pytest.mark.parametrize("name,ov", SMALL)
def test_bf16_dense_small(name, ov, qb):
    _check_dense(W.make_workload(name, dense=True, **ov), qb=qb)


@pytest.mark.parametrize("N", [1, 100, 256, 700])
@pytest.mark.parametrize("causal", [False, True])
def test_bf16_head_dim_16(N, causal):
    """C = 16 (the PDE-solver head dimension): 32-byte rows in memory, run on the 32-channel tiles."""
    w = W.make_workload("long_train", dense=True, B=2, H=2, N=N, C=16, R=8, causal=causal)
    for qb in (1, 2):
        _check_lowrank(w, qb=qb)
        _check_dense(w, qb=qb)
    _check_lowrank(W.make_workload("long_train", B=1, H=2, N=N, C=16, R=0, causal=causal))
    _check_lowrank(W.make_workload("long_train", B=1, H=2, N=N, C=16, R=5, causal=causal))


@pytest.mark.parametrize("N", [1, 33, 100, 256, 257, 383, 384])
def test_bf16_short_c32_automatic_choice(N):
    """C = 32, N <= 384, non-causal: the automatic choice is the direct-to-LDS kernel where it
    takes the shape (whole 16-byte factor rows, N % 32 == 0 for a dense bias) and the four-wave
    kernel otherwise; both must give the oracle's result."""
    for R, phi_dtype in ((16, "bf16"), (8, "bf16"), (5, "bf16"), (0, "bf16"), (2, "f32")):
        w = W.make_workload("long_train", dense=True, B=2, H=2, N=N, C=32, R=R, phi_dtype=phi_dtype)
        _check_lowrank(w)
        if R == 16:
            _check_dense(w)


@pytest.mark.parametrize("up", [0, 1])
@pytest.mark.parametrize("N", [100, 640, 1000])
def test_causal_walk_orders(N, up):
    """Both key-block orders of the causal tile pairs give the oracle's result (any order is exact
    for an online softmax; the two differ only in rounding)."""
    w = W.make_workload("alibi_causal", dense=True, B=1, H=3, N=N)
    api.fb_tune_set("fwd_causal_up", up)
    try:
        for qb in (1, 2):
            _check_lowrank(w, qb=qb)
        _check_dense(w, qb=1)
    finally:
        api.fb_tune_set("fwd_causal_up", 1)


@pytest.mark.parametrize("N", [1, 31, 64, 65])
@pytest.mark.parametrize("causal", [False, True])
def test_bf16_edge_lengths(N, causal):
    w = W.make_workload("long_train", dense=True, B=1, H=2, N=N, C=64, R=8, causal=causal)
    for qb in (1, 8, 16):
        _check_lowrank(w, qb=qb)
        _check_dense(w, qb=qb)


@pytest.mark.parametrize("C,R,phi_dtype", [(32, 64, "bf16"), (64, 0, "bf16"), (128, 48, "bf16"),
                                           (64, 10, "f32"), (128, 1, "f32"), (16, 64, "bf16"),
                                           (16, 9, "f32")])
def test_bf16_rank_range(C, R, phi_dtype):
    w = W.make_workload("long_train", B=1, H=2, N=320, C=C, R=R, phi_dtype=phi_dtype)
    _check_lowrank(w, qb=1)
    _check_lowrank(w, qb=2)
    _check_lowrank(w, qb=8)
    _check_lowrank(w, qb=16)


def test_row_shift_invariance_on_gpu():
    """A rank-1 factor c_i * 1 must leave out unchanged and add c_i to lse (exercises the
    factor columns of the contraction independently of the oracle's values)."""
    w = W.make_workload("long_train", B=1, H=2, N=256, C=64, R=0)
    d = workload_to_device(w)
    out0, lse0 = api.fb_lowrank_attn_fwd(d["q"], d["k"], d["v"], None, None)
    rng = np.random.default_rng(5)
    shift = W.round_bf16(3 * rng.standard_normal((1, 2, 256, 1)).astype(np.float32))
    pq = dev(shift, "bf16")
    pk = dev(np.ones((1, 2, 256, 1), np.float32), "bf16")
    out1, lse1 = api.fb_lowrank_attn_fwd(d["q"], d["k"], d["v"], pq, pk)
    torch.cuda.synchronize()
    assert max_abs(host(out1), host(out0)) <= 2e-2
    assert max_abs(host(lse1), host(lse0) + shift[..., 0]) <= 2e-2


def test_alibi_fp32_factors_beat_bf16_factors():
    """fp32 factors (limb-split in the kernel) reproduce ALiBi; the same factors rounded to
    bf16 do not (positions above 256 are not representable) — reported, and the first gated."""
    w = W.make_workload("alibi_causal", B=1, H=2, N=2048)
    d = workload_to_device(w)
    out, _ = api.fb_lowrank_attn_fwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], causal=True)
    wb = W.make_workload("alibi_causal", B=1, H=2, N=2048, phi_dtype="bf16")
    db = workload_to_device(wb)
    outb, _ = api.fb_lowrank_attn_fwd(db["q"], db["k"], db["v"], db["phi_q"], db["phi_k"], causal=True)
    torch.cuda.synchronize()
    slopes = O.alibi_slopes(2)
    h = 1
    rows = [5, 700, 1500, 2047]
    for r in rows:
        bias = O.alibi_bias(slopes[h], 2048)[r:r + 1]
        ref, _ = O.attention_with_bias(w.q[0, h, r:r + 1], w.k[0, h], w.v[0, h], bias, causal=True, row_offset=r)
        e32 = max_abs(host(out)[0, h, r], ref[0])
        e16 = max_abs(host(outb)[0, h, r], ref[0])
        print(f"row {r}: true-ALiBi error fp32 factors {e32:.3e}, bf16 factors {e16:.3e}", flush=True)
        assert e32 <= 2e-2
