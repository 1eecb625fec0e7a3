#!/usr/bin/env python3
"""Benchmark of the low-rank-bias attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-extras]

A step is one forward of fb_lowrank_attn_fwd over the workload (inputs resident in HBM).
Prints ONE JSON line: the headline metric (forward TFLOP/s of the low-rank kernel, algorithmic
flop 2(2C+R) per visible query-key pair), a `roofline` object for that kernel (HIP-event
duration per launch on the launch stream against the bf16 dense MFMA peak), a `cpu_baseline`
object (the float64 oracle timed on a bounded sample on this machine's host cores), and, unless
--no-extras, the dense-bias baseline, the backward and the other workloads as extra fields.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
HEADLINE = "alibi_causal"
PAPER_CONTEXT = ("paper (A100, other hardware, context only): >2x fwd vs best dense-bias "
                 "implementation for vision/language attention, 1.5x Pairformer end to end")


def _traffic_from_profile(workload: str):
    """HBM bytes per launch measured offline with rocprofv3 --pmc (see profiles/)."""
    path = os.path.join(ROOT, "profiles", f"fwd_lowrank_{workload}_hbm_traffic.txt")
    try:
        with open(path) as f:
            m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", f.read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--no-extras", action="store_true", help="headline kernel only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--probe", action="store_true",
                    help="counter-collection mode: 3 launches each of the low-rank forward, the dense "
                         "forward and the low-rank backward plus one 1 GiB device copy (calibration), "
                         "no timing output")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (see DESIGN.md, "
              "'How the path would shard'); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2505_12044_amd import api, workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    api.load_library()   # fails loudly if the HIP library is missing
    stream = torch.cuda.current_stream()

    def dev(x, name):
        t = torch.from_numpy(np.ascontiguousarray(x)).to("cuda")
        return t.to(torch.float32 if name == "f32" else torch.bfloat16).contiguous()

    def to_device(w, dense=False):
        d = dict(q=dev(w.q, w.dtype), k=dev(w.k, w.dtype), v=dev(w.v, w.dtype),
                 phi_q=dev(w.phi_q, w.phi_dtype), phi_k=dev(w.phi_k, w.phi_dtype))
        d["out"] = torch.empty_like(d["q"])
        d["lse"] = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
        if w.dout is not None:
            d["dout"] = dev(w.dout, w.dtype)
        if dense:
            if w.bias is not None:
                d["bias"] = dev(w.bias, w.dtype)
            else:   # long_train: 8.6 GB, materialised on the device from the same factors
                pq, pk = d["phi_q"].float(), d["phi_k"].float()
                d["bias"] = torch.empty((w.B, w.H, w.N, w.N), dtype=d["q"].dtype, device="cuda")
                for b in range(w.B):
                    for h in range(w.H):
                        d["bias"][b, h] = (pq[b, h] @ pk[b, h].T).to(d["q"].dtype)
        return d

    def time_calls(fn, steps, warmup):
        """Per-launch HIP-event timing on the launch stream; returns (total wall ms between
        synchronisations, mean event ms per launch)."""
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        ends = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        t0 = time.perf_counter()
        for i in range(steps):
            starts[i].record(stream)
            fn()
            ends[i].record(stream)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        ev = [s.elapsed_time(e) for s, e in zip(starts, ends)]
        return wall_ms, float(np.mean(ev))

    # ------------------------------------------------------------------ headline workload
    if args.probe:
        args.no_extras = False
    w = W.make_workload(args.workload, dense=not args.no_extras and args.workload != "long_train",
                        with_dout=not args.no_extras)
    d = to_device(w, dense=not args.no_extras)

    def fwd():
        api.fb_lowrank_attn_fwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], out=d["out"],
                                lse=d["lse"], causal=w.causal, stream=stream)

    if args.probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()   # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            fwd()
        for _ in range(3):
            api.fb_dense_bias_attn_fwd(d["q"], d["k"], d["v"], d["bias"], out=d["out"], lse=d["lse"],
                                       causal=w.causal, stream=stream)
        if "dout" in d:
            wsb = torch.empty(max(16, api.fb_lowrank_attn_bwd_workspace_bytes(w.B, w.H, w.N, w.C, w.R)),
                              dtype=torch.uint8, device="cuda")
            fwd()
            for _ in range(3):
                api.fb_lowrank_attn_bwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], d["out"], d["lse"],
                                        d["dout"], causal=w.causal, workspace=wsb, stream=stream)
        dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"probe": w.name, "copy_bytes_read": src.numel() * 4,
                          "copy_bytes_written": src.numel() * 4}))
        return 0

    wall_ms, kern_ms = time_calls(fwd, args.steps, args.warmup)
    ms_per_step = wall_ms / args.steps
    flops = w.fwd_flops()
    tflops = flops / (ms_per_step * 1e-3) / 1e12
    kern_tflops = flops / (kern_ms * 1e-3) / 1e12

    result = {
        "metric": "low-rank-bias attention fwd TFLOP/s",
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "N": w.N, "C": w.C, "R": w.R,
                   "causal": w.causal, "phi_dtype": w.phi_dtype,
                   "flop_per_pair": 2 * (2 * w.C + w.R), "pairs": w.pairs},
        "pct_of_bf16_mfma_peak": round(100 * tflops / PEAK_BF16_TFLOPS, 2),
        "roofline": {
            "kernel": "low-rank bf16 forward (fwd_bf16_kernel; fwd_bf16_pp_kernel for long non-causal sequences)",
            "bound": "mfma",
            "achieved": round(kern_tflops, 2),
            "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(kern_tflops / PEAK_BF16_TFLOPS, 4),
            "ms_per_launch": round(kern_ms, 5),
            "traffic": _traffic_from_profile(w.name),
        },
        "context": PAPER_CONTEXT,
    }

    # ------------------------------------------------------------------ extras
    if not args.no_extras:
        def dense():
            api.fb_dense_bias_attn_fwd(d["q"], d["k"], d["v"], d["bias"], out=d["out"], lse=d["lse"],
                                       causal=w.causal, stream=stream)
        n = max(10, args.steps // 4)
        _, dense_ms = time_calls(dense, n, 3)
        result["dense_bias"] = {
            "ms": round(dense_ms, 5),
            "bias_GBps": round(w.pairs * 2 / (dense_ms * 1e-3) / 1e9, 1),
            "pct_of_hbm_peak": round(100 * w.pairs * 2 / (dense_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 2),
            "speedup_lowrank_vs_dense": round(dense_ms / kern_ms, 3),
        }
        dense_bwd_ms = None
        if w.N % 8 == 0 and "dout" in d:
            # training-side baseline: dense-bias backward, which has to write the N x N bias gradient
            wsd = torch.empty(max(16, api.fb_dense_bias_attn_bwd_workspace_bytes(w.B, w.H, w.N, w.C)),
                              dtype=torch.uint8, device="cuda")
            gd = (torch.empty_like(d["q"]), torch.empty_like(d["q"]), torch.empty_like(d["q"]),
                  torch.empty((w.B, w.H, w.N, w.N), dtype=d["q"].dtype, device="cuda"))
            dense()

            def dense_bwd():
                api.fb_dense_bias_attn_bwd(d["q"], d["k"], d["v"], d["bias"], d["out"], d["lse"], d["dout"],
                                           causal=w.causal, workspace=wsd, grads=gd, stream=stream)
            _, dense_bwd_ms = time_calls(dense_bwd, max(5, n // 2), 2)
            del gd, wsd
        d.pop("bias", None)
        torch.cuda.empty_cache()

        if w.name == "alibi_causal":
            # the same bias generated inside the kernel from the head slopes (no factor loads)
            from paper_2505_12044_amd.workloads import alibi_slopes_f32
            slopes = torch.from_numpy(alibi_slopes_f32(w.H)).cuda()

            def jit():
                api.fb_alibi_attn_fwd(d["q"], d["k"], d["v"], slopes, out=d["out"], lse=d["lse"],
                                      causal=w.causal, stream=stream)
            _, jit_ms = time_calls(jit, n, 3)
            result["alibi_in_kernel"] = {
                "ms": round(jit_ms, 5),
                "TFLOPs": round(flops / (jit_ms * 1e-3) / 1e12, 2),
                "vs_factor_tensors": round(kern_ms / jit_ms, 3),
            }
            if "dout" in d:
                wsj = torch.empty(api.fb_alibi_attn_bwd_workspace_bytes(w.B, w.H, w.N, w.C), dtype=torch.uint8,
                                  device="cuda")
                gj = (torch.empty_like(d["q"]), torch.empty_like(d["q"]), torch.empty_like(d["q"]))
                jit()

                def jit_bwd():
                    api.fb_alibi_attn_bwd(d["q"], d["k"], d["v"], slopes, d["out"], d["lse"], d["dout"],
                                          causal=w.causal, workspace=wsj, grads=gj, stream=stream)
                _, jit_bwd_ms = time_calls(jit_bwd, n, 3)
                result["alibi_in_kernel"]["bwd_ms"] = round(jit_bwd_ms, 5)
                del wsj, gj

        ws = torch.empty(max(16, api.fb_lowrank_attn_bwd_workspace_bytes(w.B, w.H, w.N, w.C, w.R)),
                         dtype=torch.uint8, device="cuda")
        grads = (torch.empty_like(d["q"]), torch.empty_like(d["q"]), torch.empty_like(d["q"]),
                 torch.empty((w.B, w.H, w.N, w.R), dtype=d["phi_q"].dtype, device="cuda"),
                 torch.empty((w.B, w.H, w.N, w.R), dtype=d["phi_q"].dtype, device="cuda"))

        def bwd():
            api.fb_lowrank_attn_bwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], d["out"], d["lse"],
                                    d["dout"], causal=w.causal, workspace=ws, grads=grads, stream=stream)
        fwd()
        _, bwd_ms = time_calls(bwd, n, 3)
        result["backward"] = {"ms": round(bwd_ms, 5),
                              "TFLOPs": round(w.bwd_flops() / (bwd_ms * 1e-3) / 1e12, 2)}
        if dense_bwd_ms is not None:
            result["backward"]["dense_bias_ms"] = round(dense_bwd_ms, 5)
            result["backward"]["speedup_lowrank_vs_dense"] = round(dense_bwd_ms / bwd_ms, 3)
            result["backward"]["dense_dbias_bytes"] = int(w.B * w.H * w.N * w.N * 2)
        del grads, ws

        others = {}
        for name in W.CONFIG_NAMES:
            if name in (w.name, "tiny_fp32"):
                continue
            del d
            torch.cuda.empty_cache()
            wo = W.make_workload(name, dense=name != "long_train", with_dout=name == "long_train")
            d = to_device(wo, dense=True)
            w_ = wo

            def f2():
                api.fb_lowrank_attn_fwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], out=d["out"],
                                        lse=d["lse"], causal=w_.causal, stream=stream)

            def d2():
                api.fb_dense_bias_attn_fwd(d["q"], d["k"], d["v"], d["bias"], out=d["out"], lse=d["lse"],
                                           causal=w_.causal, stream=stream)
            # short kernels: enough untimed launches for the clocks to settle
            wu = 100 if wo.pairs < (1 << 32) else 3
            _, ms_lr = time_calls(f2, n, wu)
            _, ms_de = time_calls(d2, max(5, n // 2), wu)
            row = {"B": wo.B, "H": wo.H, "N": wo.N, "C": wo.C, "R": wo.R,
                   "fwd_ms": round(ms_lr, 5),
                   "fwd_TFLOPs": round(wo.fwd_flops() / (ms_lr * 1e-3) / 1e12, 2),
                   "pct_of_bf16_mfma_peak": round(100 * wo.fwd_flops() / (ms_lr * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2),
                   "dense_ms": round(ms_de, 5),
                   "dense_bias_GBps": round(wo.pairs * 2 / (ms_de * 1e-3) / 1e9, 1),
                   "speedup_lowrank_vs_dense": round(ms_de / ms_lr, 3)}
            if name == "long_train":
                f_ms_db = None
                if wo.N % 8 == 0:
                    wsd = torch.empty(api.fb_dense_bias_attn_bwd_workspace_bytes(wo.B, wo.H, wo.N, wo.C),
                                      dtype=torch.uint8, device="cuda")
                    gd = (torch.empty_like(d["q"]), torch.empty_like(d["q"]), torch.empty_like(d["q"]),
                          torch.empty((wo.B, wo.H, wo.N, wo.N), dtype=d["q"].dtype, device="cuda"))
                    d2()

                    def db2():
                        api.fb_dense_bias_attn_bwd(d["q"], d["k"], d["v"], d["bias"], d["out"], d["lse"],
                                                   d["dout"], causal=w_.causal, workspace=wsd, grads=gd,
                                                   stream=stream)
                    _, f_ms_db = time_calls(db2, 3, 1)
                    del gd, wsd
                d.pop("bias", None)
                torch.cuda.empty_cache()
                ws = torch.empty(api.fb_lowrank_attn_bwd_workspace_bytes(wo.B, wo.H, wo.N, wo.C, wo.R),
                                 dtype=torch.uint8, device="cuda")
                f2()

                def b2():
                    api.fb_lowrank_attn_bwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], d["out"],
                                            d["lse"], d["dout"], causal=w_.causal, workspace=ws,
                                            stream=stream)
                _, ms_b = time_calls(b2, 5, 1)
                row["bwd_ms"] = round(ms_b, 4)
                row["bwd_TFLOPs"] = round(wo.bwd_flops() / (ms_b * 1e-3) / 1e12, 2)
                if f_ms_db is not None:
                    row["dense_bwd_ms"] = round(f_ms_db, 4)
                    row["bwd_speedup_lowrank_vs_dense"] = round(f_ms_db / ms_b, 3)
                    row["dense_dbias_bytes"] = int(wo.B * wo.H * wo.N * wo.N * 2)
            others[name] = row
        # the PDE-solver shape (Sec. 4.3): ragged N, head dimension 16, rank-9 fp32 distance factors
        del d
        torch.cuda.empty_cache()
        wp = W.make_pde_workload()
        d = to_device(wp)
        ws = torch.empty(api.fb_lowrank_attn_bwd_workspace_bytes(wp.B, wp.H, wp.N, wp.C, wp.R),
                         dtype=torch.uint8, device="cuda")

        def f3():
            api.fb_lowrank_attn_fwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], out=d["out"],
                                    lse=d["lse"], stream=stream)

        def b3():
            api.fb_lowrank_attn_bwd(d["q"], d["k"], d["v"], d["phi_q"], d["phi_k"], d["out"], d["lse"],
                                    d["dout"], workspace=ws, stream=stream)
        _, ms_f = time_calls(f3, 10, 2)
        _, ms_b = time_calls(b3, 5, 1)
        others["pde_distance"] = {
            "B": wp.B, "H": wp.H, "N": wp.N, "C": wp.C, "R": wp.R, "phi_dtype": "f32",
            "fwd_ms": round(ms_f, 4), "fwd_TFLOPs": round(wp.fwd_flops() / (ms_f * 1e-3) / 1e12, 2),
            "bwd_ms": round(ms_b, 4), "bwd_TFLOPs": round(wp.bwd_flops() / (ms_b * 1e-3) / 1e12, 2),
            "dense_bias_bytes_avoided": int(wp.H * wp.N * wp.N * 2)}
        del ws, d
        torch.cuda.empty_cache()
        # the same bias as five merged columns (|x|^2 + |y|^2 - 2 x.y): padded factor width 32 instead of 64
        wp5 = W.make_pde_workload(rank5=True)
        d = to_device(wp5)
        ws = torch.empty(api.fb_lowrank_attn_bwd_workspace_bytes(wp5.B, wp5.H, wp5.N, wp5.C, wp5.R),
                         dtype=torch.uint8, device="cuda")
        _, ms_f5 = time_calls(f3, 10, 2)
        _, ms_b5 = time_calls(b3, 5, 1)
        others["pde_distance"]["rank5_fwd_ms"] = round(ms_f5, 4)
        others["pde_distance"]["rank5_bwd_ms"] = round(ms_b5, 4)
        del ws, d
        torch.cuda.empty_cache()

        # multiplicative bias cos(i - j) as rank-2 factors (App. I): pre-pass + forward on 2C channels
        Bm, Hm, Nm, Cm = 4, 16, 4096, 64
        g = torch.Generator(device="cuda").manual_seed(1007)
        qm, km, vm = (torch.randn((Bm, Hm, Nm, Cm), device="cuda", generator=g).to(torch.bfloat16) for _ in range(3))
        pos = torch.arange(Nm, device="cuda", dtype=torch.float64)
        fm = torch.stack([torch.cos(pos), torch.sin(pos)], dim=1).to(torch.float32)
        fm = fm.expand(1, Hm, Nm, 2).contiguous()
        om = torch.empty_like(qm)
        lm = torch.empty((Bm, Hm, Nm), dtype=torch.float32, device="cuda")
        wsm = torch.empty(api.fb_lowrank_mulbias_attn_fwd_workspace_bytes(Bm, Hm, Nm, Cm, 2), dtype=torch.uint8,
                          device="cuda")

        def fm_():
            api.fb_lowrank_mulbias_attn_fwd(qm, km, vm, fm, fm, out=om, lse=lm, workspace=wsm, stream=stream)

        def plain():
            api.fb_lowrank_attn_fwd(qm, km, vm, None, None, out=om, lse=lm, stream=stream)
        _, ms_m = time_calls(fm_, 10, 2)
        _, ms_p = time_calls(plain, 10, 2)
        dom = torch.randn((Bm, Hm, Nm, Cm), device="cuda", generator=g).to(torch.bfloat16)
        wsb = torch.empty(api.fb_lowrank_mulbias_attn_bwd_workspace_bytes(Bm, Hm, Nm, Cm, 2), dtype=torch.uint8,
                          device="cuda")
        fm_()

        def bm_():
            api.fb_lowrank_mulbias_attn_bwd(qm, km, vm, fm, fm, om, lm, dom, workspace=wsb, stream=stream)
        _, ms_mb = time_calls(bm_, 5, 1)
        del wsb, dom
        pairs_m = Bm * Hm * Nm * Nm
        others["multiplicative_cos"] = {
            "B": Bm, "H": Hm, "N": Nm, "C": Cm, "R": 2, "fwd_ms_incl_prepass": round(ms_m, 4),
            "fwd_TFLOPs": round(2.0 * (Cm * 2 + Cm) * pairs_m / (ms_m * 1e-3) / 1e12, 2),
            "plain_attention_ms": round(ms_p, 4), "cost_vs_plain": round(ms_m / ms_p, 3),
            "bwd_ms_incl_prepass_and_fold": round(ms_mb, 4),
            "dense_bias_bytes_avoided": int(Hm * Nm * Nm * 2)}
        del qm, km, vm, om, lm, wsm
        result["other_workloads"] = others

    # ------------------------------------------------------------------ CPU oracle
    if not args.no_cpu:
        from oracle import fb_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        wh = w
        heads = 0
        t0 = time.perf_counter()
        budget = 15.0     # seconds of oracle work; the (batch, head) pairs are cycled until it is spent
        n_bh = wh.B * wh.H
        while time.perf_counter() - t0 < budget:
            b, h = divmod(heads % n_bh, wh.H)
            bp = 0 if wh.phi_q.shape[0] == 1 else b
            O.attention_lowrank(wh.q[b, h], wh.k[b, h], wh.v[b, h], wh.phi_q[bp, h], wh.phi_k[bp, h],
                                causal=wh.causal)
            heads += 1
        dt = time.perf_counter() - t0
        per_head = flops / (w.B * w.H)
        result["cpu_baseline"] = {
            "value": round(heads * per_head / dt / 1e12, 5),
            "unit": "TFLOP/s",
            "cores": int(cores),
            "kind": "oracle",
            "sample": f"{heads} single-(batch, head) forwards of {w.name} ({w.B * w.H} distinct) in float64, "
                      f"{dt:.1f} s",
        }

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
