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


def err_stats(got, ref):
    """(max abs error, max abs error / RMS(ref), max |ref|) of one output tensor."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0, 0.0, 0.0
    e = float(np.max(np.abs(got - ref)))
    rms = float(np.sqrt(np.mean(ref * ref)))
    return e, (e / rms if rms > 0 else (0.0 if e == 0 else float("inf"))), float(np.max(np.abs(ref)))


def report(label, name, got, ref):
    """Prints the unscaled max-abs error and the error relative to RMS(ref) of one output, so a
    loose absolute bound cannot hide an error that is large for the data; returns both and max|ref|."""
    e, rel, big = err_stats(got, ref)
    print(f"[parity] {label} {name}: max_abs {e:.3e}  max_abs/rms(ref) {rel:.3e}  max|ref| {big:.3g}", flush=True)
    return e, rel, big


def check_fwd(label, name, got, ref, dtype="bf16"):
    """Forward outputs: flat bound of the storage type (1e-4 fp32, 2e-2 bf16), both figures printed."""
    got = np.asarray(got, np.float64)
    assert np.isfinite(got).all(), (label, name)
    e, rel, _ = report(label, name, got, ref)
    assert e <= TOL[dtype], (label, name, e)
    return e


def check_grad(label, name, got, ref, data_scaled=False, gain=1.0):
    """Gradients: flat 5e-2 max abs error unless the case is marked data_scaled (bound times
    max(1, max|ref| / 2.5): gradient entries of magnitude 10 and more, where bf16 storage of the
    result alone is 2^-9 relative) or carries a stated gain; both figures are always printed."""
    got = np.asarray(got, np.float64)
    assert np.isfinite(got).all(), (label, name)
    e, rel, big = report(label, name, got, ref)
    limit = GRAD_TOL * gain * (max(1.0, big / 2.5) if data_scaled else 1.0)
    assert e <= limit, (label, name, e, limit, "flat bound would be", GRAD_TOL)
    return e


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
