"""Tensors of 2^31 elements: offsets above the head level are 64-bit in every kernel, so the
library accepts them (the size limits are the row count and the extent of one head, see
include/flashbias.h).  B 16, H 8, N 131072, C 128, R 8: q, k, v, out hold 2^31 bf16 elements (4 GiB) each.
Inputs are drawn on the device (seeded); the rows the oracle checks are copied back.  Checked:
forward rows and dq / dphi_q rows of the first head and of the last one, whose element offsets lie
beyond 2^31 (a row of dq depends on its own query row and all keys, so the oracle's chain rule on a
slice of query rows is exact for it)."""
import numpy as np
import pytest
import torch

from oracle import fb_oracle as O
from paper_2505_12044_amd import api
from tests._gpu_util import check_fwd, check_grad, host

pytestmark = pytest.mark.gpu


def test_forward_and_backward_beyond_2_31_elements():
    B, H, N, C, R = 16, 8, 131072, 128, 8
    assert B * H * N * C == 1 << 31
    g = torch.Generator(device="cuda").manual_seed(9001)

    def draw(*shape, std=1.0):
        t = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
        for b in range(shape[0]):        # one batch item at a time bounds the fp32 temporary
            t[b] = (std * torch.randn(shape[1:], device="cuda", generator=g)).to(torch.bfloat16)
        return t

    q, k, v, dout = draw(B, H, N, C), draw(B, H, N, C), draw(B, H, N, C), draw(B, H, N, C)
    pq, pk = draw(B, H, N, R, std=R ** -0.25), draw(B, H, N, R, std=R ** -0.25)
    out, lse = api.fb_lowrank_attn_fwd(q, k, v, pq, pk)
    grads = api.fb_lowrank_attn_bwd(q, k, v, pq, pk, out, lse, dout)
    torch.cuda.synchronize()
    rng = np.random.default_rng(9002)
    for (b, h) in ((0, 0), (B - 1, H - 1)):
        kh, vh, pkh = host(k[b, h]), host(v[b, h]), host(pk[b, h])
        rows = sorted({0, 127, 128, N - 129, N - 1} | set(int(x) for x in rng.integers(0, N, 11)))
        qr, pqr, dor = host(q[b, h, rows]), host(pq[b, h, rows]), host(dout[b, h, rows])
        ro, rl = O.attention_lowrank(qr, kh, vh, pqr, pkh)
        label = f"2^31-element tensors, (b,h)=({b},{h}), {len(rows)} rows"
        check_fwd(label, "out", host(out[b, h, rows]), ro)
        check_fwd(label, "lse", host(lse[b, h, rows]), rl)
        rdq, _, _, rdpq, _ = O.attention_lowrank_grads(qr, kh, vh, pqr, pkh, dor)
        check_grad(label, "dq", host(grads[0][b, h, rows]), rdq)
        check_grad(label, "dphi_q", host(grads[3][b, h, rows]), rdpq)
    # key-side gradients of the last head: finite and not identically zero (their oracle needs all N^2 pairs)
    for name, t in (("dk", grads[1]), ("dv", grads[2]), ("dphi_k", grads[4])):
        x = t[B - 1, H - 1].float()
        assert torch.isfinite(x).all() and float(x.abs().max()) > 0, name
