"""The forward and the allocation-free backward under HIP graph capture (what the allocation-free
entry point is for): a captured forward + backward pair is replayed several times on new inputs,
with eager work and synchronisations between the replays, and every replay must equal the eager
result bit for bit."""
import pytest
import torch

from paper_2505_12044_amd import api, workloads as W
from tests._gpu_util import workload_to_device

pytestmark = pytest.mark.gpu


def test_forward_and_noalloc_backward_replay_in_a_graph():
    w = W.make_workload("long_train", with_dout=True, B=1, H=2, N=384, C=64, R=8, causal=True)
    d = workload_to_device(w)
    names = ("q", "k", "v", "phi_q", "phi_k", "dout")
    static = {n: d[n].clone() for n in names}
    out = torch.empty_like(static["q"])
    lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
    grads = (torch.empty_like(static["q"]), torch.empty_like(static["k"]), torch.empty_like(static["v"]),
             torch.empty_like(static["phi_q"].expand(w.B, -1, -1, -1).contiguous()),
             torch.empty_like(static["phi_k"].expand(w.B, -1, -1, -1).contiguous()))

    def step():
        api.fb_lowrank_attn_fwd(static["q"], static["k"], static["v"], static["phi_q"], static["phi_k"],
                                out=out, lse=lse, causal=True)
        api.fb_lowrank_attn_bwd_noalloc(static["q"], static["k"], static["v"], static["phi_q"], static["phi_k"],
                                        out, lse, static["dout"], grads, causal=True)

    # eager warm-up on a side stream: per-kernel attributes and the scratch address are set up outside the capture
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        step()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    torch.cuda.synchronize()

    gen = torch.Generator(device="cuda").manual_seed(5)
    for rep in range(3):
        fresh = {n: (torch.randn(static[n].shape, generator=gen, device="cuda") * (0.5 if "phi" in n else 1.0))
                 .to(static[n].dtype) for n in names}
        # eager reference on separate outputs
        eo, el = api.fb_lowrank_attn_fwd(fresh["q"], fresh["k"], fresh["v"], fresh["phi_q"], fresh["phi_k"], causal=True)
        eg = api.fb_lowrank_attn_bwd(fresh["q"], fresh["k"], fresh["v"], fresh["phi_q"], fresh["phi_k"], eo, el,
                                     fresh["dout"], causal=True)
        torch.cuda.synchronize()
        for n in names:
            static[n].copy_(fresh[n])
        for t in (out, lse, *grads):
            t.fill_(float("nan"))          # (a fill kernel, outside the graph)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eo) and torch.equal(lse, el), rep
        for name, a, b in zip(("dq", "dk", "dv", "dphi_q", "dphi_k"), grads, eg):
            assert torch.equal(a, b), (rep, name)
