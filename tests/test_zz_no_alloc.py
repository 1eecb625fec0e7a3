"""The allocation-free backward entry point (fb_lowrank_attn_bwd_noalloc) against the entry point
it is a variant of (fb_lowrank_attn_bwd with a caller workspace): same kernels on the library's
static device scratch, so the results must be bit-identical.  Two calls in a row, the second on
a smaller problem (the static array still holds the first call's rows), then the size limit."""
import numpy as np
import pytest
import torch

from oracle import fb_oracle as O
from paper_2505_12044_amd import api, workloads as W
from tests._gpu_util import GRAD_TOL, host, max_abs, workload_to_device

pytestmark = pytest.mark.gpu


def _both(w):
    d = workload_to_device(w)
    out, lse = api.fb_lowrank_attn_fwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], causal=w.causal)
    ref = api.fb_lowrank_attn_bwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], out, lse, d["dout"],
                                  causal=w.causal)
    grads = tuple(torch.full_like(g, float("nan")) for g in ref)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    got = api.fb_lowrank_attn_bwd_noalloc(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], out, lse, d["dout"],
                                          grads, causal=w.causal)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before     # the binding allocates nothing
    return ref, got


def test_noalloc_backward_matches_workspace_backward_twice():
    big = W.make_workload("long_train", with_dout=True, B=2, H=4, N=1000, R=8)            # ragged, 8000 rows
    small = W.make_workload("alibi_causal", with_dout=True, B=1, H=2, N=333)              # fp32 factors, causal
    for w in (big, small):
        need = api.fb_lowrank_attn_bwd_workspace_bytes(w.B, w.H, w.N, w.C, w.R)
        assert need <= api.FB_STATIC_SCRATCH_BYTES
        ref, got = _both(w)
        for name, a, b in zip(("dq", "dk", "dv", "dphi_q", "dphi_k"), ref, got):
            assert torch.isfinite(b.float()).all(), name
            assert torch.equal(a, b), (w.name, name)
    # and against the oracle, to the usual gradient bound, for the second (smaller) call
    r = O.batched_attention_lowrank_grads(small.q, small.k, small.v, small.phi_q, small.phi_k, small.dout, causal=True)
    for name, g, x in zip(("dq", "dk", "dv"), got, r):
        err = max_abs(host(g), x)
        print(f"noalloc {name}: max abs err {err:.3e} (max|ref| {np.abs(x).max():.2f})", flush=True)
        assert err <= GRAD_TOL * max(1.0, float(np.abs(x).max()) / 2.5)


def test_noalloc_backward_rejects_oversize():
    lib = api.load_library()
    B, H, N, C, R = 4, 16, 4096, 128, 2
    assert api.fb_lowrank_attn_bwd_workspace_bytes(B, H, N, C, R) > api.FB_STATIC_SCRATCH_BYTES
    x = torch.zeros(16, dtype=torch.bfloat16, device="cuda")      # never touched: the call must fail before any launch
    p = x.data_ptr()
    st = lib.fb_lowrank_attn_bwd_noalloc(p, p, p, p, p, p, p, p, p, p, p, p, p, B, H, N, C, R, 1, api.FB_BF16,
                                         api.FB_F32, 1, 0.0, None)
    assert st == 7 and b"static scratch" in lib.fb_status_string(st)
