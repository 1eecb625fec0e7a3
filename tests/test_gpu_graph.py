"""The entry points only enqueue kernels on the caller's stream (no allocation, no
synchronisation, no memset), so a forward + backward step can be captured into a HIP graph.
The graph is replayed several times with eager work and synchronisations in between, and every
replay is compared with the eager result."""
import numpy as np
import pytest
import torch

from paper_2505_12044_amd import api, workloads as W
from tests._gpu_util import dev

pytestmark = pytest.mark.gpu


def test_forward_backward_graph_replay():
    w = W.make_workload("long_train", with_dout=True, B=1, H=2, N=640)
    q, k, v, do = (dev(x, "bf16") for x in (w.q, w.k, w.v, w.dout))
    pq, pk = dev(w.phi_q, "bf16"), dev(w.phi_k, "bf16")
    out = torch.empty_like(q)
    lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
    ws = torch.empty(api.fb_lowrank_attn_bwd_workspace_bytes(w.B, w.H, w.N, w.C, w.R), dtype=torch.uint8,
                     device="cuda")
    grads = (torch.empty_like(q), torch.empty_like(q), torch.empty_like(q), torch.empty_like(pq),
             torch.empty_like(pk))

    def step(stream=None):
        api.fb_lowrank_attn_fwd(q, k, v, pq, pk, out=out, lse=lse, stream=stream)
        api.fb_lowrank_attn_bwd(q, k, v, pq, pk, out, lse, do, workspace=ws, grads=grads, stream=stream)

    step()                              # eager reference (also sets the kernels' launch attributes)
    torch.cuda.synchronize()
    ref = [t.clone() for t in (out, lse) + grads]

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(torch.cuda.current_stream())
    for rep in range(3):
        for t in (out, lse) + grads:
            t.zero_()                   # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip((out, lse) + grads, ref):
            assert torch.equal(a, b), f"replay {rep} differs from the eager result"


def test_other_entry_points_graph_replay():
    """In-kernel ALiBi forward, dense-bias forward, multiplicative forward + backward (pre-pass,
    main kernels, fold) in one captured graph."""
    B, H, N, C = 1, 2, 384, 64
    rng = np.random.default_rng(9900)
    q, k, v, do = (dev(W.round_bf16(rng.standard_normal((B, H, N, C)).astype(np.float32)), "bf16") for _ in range(4))
    slopes = torch.tensor([0.25, 0.0625], dtype=torch.float32, device="cuda")
    bias = dev(W.round_bf16(rng.standard_normal((1, H, N, N)).astype(np.float32)), "bf16")
    f = dev(rng.uniform(-1, 1, (1, H, N, 2)).astype(np.float32), "f32")
    outs = [torch.empty_like(q) for _ in range(3)]
    lses = [torch.empty((B, H, N), dtype=torch.float32, device="cuda") for _ in range(3)]
    ws_f = torch.empty(api.fb_lowrank_mulbias_attn_fwd_workspace_bytes(B, H, N, C, 2), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(api.fb_lowrank_mulbias_attn_bwd_workspace_bytes(B, H, N, C, 2), dtype=torch.uint8, device="cuda")
    grads = (torch.empty_like(q), torch.empty_like(q), torch.empty_like(q),
             torch.empty((B, H, N, 2), dtype=torch.float32, device="cuda"),
             torch.empty((B, H, N, 2), dtype=torch.float32, device="cuda"))

    def step(stream=None):
        api.fb_alibi_attn_fwd(q, k, v, slopes, out=outs[0], lse=lses[0], causal=True, stream=stream)
        api.fb_dense_bias_attn_fwd(q, k, v, bias, out=outs[1], lse=lses[1], stream=stream)
        api.fb_lowrank_mulbias_attn_fwd(q, k, v, f, f, out=outs[2], lse=lses[2], workspace=ws_f, stream=stream)
        api.fb_lowrank_mulbias_attn_bwd(q, k, v, f, f, outs[2], lses[2], do, workspace=ws_b, grads=grads,
                                        stream=stream)

    step()
    torch.cuda.synchronize()
    allt = tuple(outs) + tuple(lses) + grads
    ref = [t.clone() for t in allt]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(torch.cuda.current_stream())
    for rep in range(3):
        for t in allt:
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(allt, ref):
            assert torch.equal(a, b), f"replay {rep} differs from the eager result"
