"""Helpers shared by the GPU parity tests: host arrays -> device buffers, oracle calls."""
import numpy as np
import torch

from oracle import fb_oracle as O

TOL = {"f32": 1e-4, "bf16": 2e-2}
GRAD_TOL = 5e-2


def tdtype(name):
    return torch.float32 if name == "f32" else torch.bfloat16


def dev(x, dtype_name):
    """float32 host array holding storage-exact values -> CUDA tensor of that storage type."""
    if x is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda").to(tdtype(dtype_name)).contiguous()


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def workload_to_device(w, dense=False):
    d = dict(q=dev(w.q, w.dtype), k=dev(w.k, w.dtype), v=dev(w.v, w.dtype),
             phi_q=dev(w.phi_q, w.phi_dtype) if w.R else None,
             phi_k=dev(w.phi_k, w.phi_dtype) if w.R else None)
    if w.dout is not None:
        d["dout"] = dev(w.dout, w.dtype)
    if dense and w.bias is not None:
        d["bias"] = dev(w.bias, w.dtype)
    return d


def max_abs(a, b):
    return float(np.max(np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64)))) if np.size(a) else 0.0


def oracle_rows_lowrank(w, b, h, rows):
    """Oracle out/lse for the given query rows of one (b, h) at full key length."""
    bp = 0 if w.phi_q.shape[0] == 1 else b
    outs, lses = [], []
    for r in rows:
        o, l = O.attention_lowrank(w.q[b, h, r:r + 1], w.k[b, h], w.v[b, h],
                                   w.phi_q[bp, h, r:r + 1], w.phi_k[bp, h],
                                   causal=w.causal, row_offset=int(r))
        outs.append(o[0]); lses.append(l[0])
    return np.array(outs), np.array(lses)
