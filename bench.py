#!/usr/bin/env python3
"""Benchmark of the low-rank-bias attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-extras] [--no-cpu]

A step is one forward of fb_lowrank_attn_fwd over the workload (inputs resident in HBM).
Prints ONE JSON line: the headline metric (forward TFLOP/s of the low-rank kernel, algorithmic
flop 2(2C+R) per visible query-key pair), a `roofline` object for that kernel (HIP-event
duration per launch on the launch stream against the bf16 dense MFMA peak, plus the ceiling a
bare MFMA loop reaches on this chip), a `cpu_baseline` object (the float64 oracle timed on a
bounded sample on this machine's host cores), and, unless --no-extras, the dense-bias baseline, the
backward and the other workloads as extra fields.

Timing protocol.  Before anything is timed the kernel is launched back to back for
`settle_s` seconds (untimed): the chip raises its clocks only under sustained load, and a
short run otherwise measures the ramp (0.37 ms against 0.31 ms per launch on the headline
workload).  Then W warm-up steps, then exactly K steps between two synchronisations
(`ms_per_step`, `value`).  Kernel-level figures are the median of five repeats, each the mean
HIP-event duration of its launches.  Workloads whose working set fits the 256 MB Infinity
Cache are also timed "cold": the launches rotate over copies of every tensor that together
exceed 512 MB, so no launch finds its inputs in cache.
"""
from __future__ import annotations

import argparse
import ctypes
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
# fp32 vector rate without packed operations: 256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz
PEAK_VALU_TFLOPS = 78.6
# vector work of the softmax per (query, key) pair, in fp32-flop equivalents: one multiply-add (2),
# one exponential at a quarter of the vector rate (4), conversion to bf16 and row sum (2)
SOFTMAX_FLOP_PER_PAIR = 8
HEADLINE = "alibi_causal"
SETTLE_S = 0.3
REPEATS = 5
COLD_BYTES = 512 << 20
PAPER_CONTEXT = ("paper (A100, other hardware, context only): >2x fwd vs best dense-bias "
                 "implementation for vision/language attention, 1.5x Pairformer end to end")


def _profile_field(path_stem: str, field: str):
    """A figure measured offline with rocprofv3 --pmc and kept in profiles/ (None when absent)."""
    path = os.path.join(ROOT, "profiles", path_stem)
    try:
        with open(path) as f:
            m = re.search(rf"^{field}:\s*([0-9.eE+]+)", f.read(), re.M)
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
        print("bench.py measures one GPU: this build has no multi-GPU path (attention shards over "
              "batch and heads with no communication); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2505_12044_amd import api, build as fb_build, workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    api.load_library()   # fails loudly if the HIP library is missing
    stream = torch.cuda.current_stream()
    probe = None
    if os.path.exists(fb_build.PROBE_LIB):
        probe = ctypes.CDLL(fb_build.PROBE_LIB)
        probe.fbp_mfma_loop.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        probe.fbp_mfma_loop_flop.restype = ctypes.c_double
        probe.fbp_mfma_loop_flop.argtypes = [ctypes.c_int, ctypes.c_int]
        probe.fbp_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]

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

    def stream_handle():
        return stream.cuda_stream or None

    # ------------------------------------------------------------------ timing helpers
    def settle(fn, seconds=SETTLE_S):
        """Untimed back-to-back launches for `seconds`: brings the clocks to their loaded state."""
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            for _ in range(20):
                fn()
            torch.cuda.synchronize()

    def timed_region(fn, steps, events=True):
        """Exactly `steps` launches between two synchronisations.  With events: per-launch HIP events on
        the launch stream (two more packets per launch, which widen the gaps between kernels by a few
        microseconds, so the contract's wall-clock region runs without them).  Returns (wall ms of the
        region, mean event ms per launch or None)."""
        if events:
            starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
            ends = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            if events:
                starts[i].record(stream)
            fn()
            if events:
                ends[i].record(stream)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        if not events:
            return wall_ms, None
        return wall_ms, float(np.mean([s.elapsed_time(e) for s, e in zip(starts, ends)]))

    def kernel_ms(fn, steps=None, repeats=REPEATS, do_settle=True):
        """Median over `repeats` of the mean event duration of `steps` launches (steps chosen so that
        one repeat lasts about 0.1 s when not given)."""
        if do_settle:
            settle(fn)
        if steps is None:
            _, est = timed_region(fn, 3)
            steps = int(min(100, max(3, 100.0 / max(est, 1e-3))))
        vals = [timed_region(fn, steps)[1] for _ in range(repeats)]
        return float(np.median(vals)), steps

    def rotating(make_call, tensors, bytes_per_set):
        """Cold-cache variant of a launch: copies of the tensors that together exceed COLD_BYTES,
        visited round-robin, so no launch finds its operands in the 256 MB Infinity Cache."""
        nset = int(max(2, -(-COLD_BYTES // max(1, bytes_per_set)) + 1))
        sets = [tensors] + [{k: (v.clone() if torch.is_tensor(v) else v) for k, v in tensors.items()}
                            for _ in range(nset - 1)]
        state = {"i": 0}

        def call():
            make_call(sets[state["i"]])
            state["i"] = (state["i"] + 1) % nset
        return call, nset, sets

    def tensor_bytes(d):
        return int(sum(v.numel() * v.element_size() for v in d.values() if torch.is_tensor(v)))

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
        nbytes = 1 << 30
        src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").normal_()
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
        if probe is not None:
            probe.fbp_copy(src.data_ptr(), dst.data_ptr(), nbytes, stream_handle())
        else:
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"probe": w.name, "copy_bytes_read": nbytes, "copy_bytes_written": nbytes,
                          "copy_kernel": "copy_kernel (fbp_copy)" if probe is not None else "torch copy_"}))
        return 0

    settle(fwd)
    for _ in range(args.warmup):
        fwd()
    wall_ms, _ = timed_region(fwd, args.steps, events=False)   # the contract's timed region: exactly K steps
    ms_per_step = wall_ms / args.steps
    reps = [timed_region(fwd, args.steps)[1] for _ in range(REPEATS)]
    kern_ms = float(np.median(reps))
    flops = w.fwd_flops()
    tflops = flops / (ms_per_step * 1e-3) / 1e12
    kern_tflops = flops / (kern_ms * 1e-3) / 1e12

    ceiling = None
    if probe is not None:
        blocks, iters = 512, 4000         # two workgroups per CU: two waves per SIMD; ~2 ms per launch
        buf = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")

        def mfma_loop():
            probe.fbp_mfma_loop(buf.data_ptr(), blocks, iters, stream_handle())
        c_ms, _ = kernel_ms(mfma_loop, steps=20)     # settled like every other kernel: sustained rate
        ceiling = probe.fbp_mfma_loop_flop(blocks, iters) / (c_ms * 1e-3) / 1e12

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
        "settle_s": SETTLE_S,
        "pct_of_bf16_mfma_peak": round(100 * tflops / PEAK_BF16_TFLOPS, 2),
        "roofline": {
            "kernel": "low-rank bf16 forward (fwd_bf16_kernel, four waves per workgroup)",
            "bound": "mfma",
            "achieved": round(kern_tflops, 2),
            "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(kern_tflops / PEAK_BF16_TFLOPS, 4),
            "ms_per_launch": round(kern_ms, 5),
            "ms_per_launch_repeats": [round(x, 5) for x in reps],
            "traffic": _profile_field(f"fwd_lowrank_{w.name}_hbm_traffic.txt", "traffic_bytes_per_launch"),
        },
        "context": PAPER_CONTEXT,
    }
    if ceiling is not None:
        result["roofline"]["measured_ceiling"] = round(ceiling, 1)
        result["roofline"]["measured_ceiling_kernel"] = ("back-to-back v_mfma_f32_32x32x16_bf16, two waves per "
                                                         "SIMD, no memory traffic (libfb_bench_probe.so)")
        result["roofline"]["frac_of_measured_ceiling"] = round(kern_tflops / ceiling, 4)

    # ------------------------------------------------------------------ extras
    if not args.no_extras:
        def unique_bias_bytes(wl):
            per = wl.N * (wl.N + 1) // 2 if wl.causal else wl.N * wl.N
            bb = 1 if (wl.bias is not None and wl.bias.shape[0] == 1) else wl.B
            return bb * wl.H * per * 2

        def dense():
            api.fb_dense_bias_attn_fwd(d["q"], d["k"], d["v"], d["bias"], out=d["out"], lse=d["lse"],
                                       causal=w.causal, stream=stream)
        dense_ms, _ = kernel_ms(dense)
        result["dense_bias"] = {
            "ms": round(dense_ms, 5),
            # bytes of distinct bias entries the launch has to fetch at least once (a bias shared over the
            # batch counts once), over the launch time: a lower bound on the HBM rate, not a counter
            "unique_bias_bytes": unique_bias_bytes(w),
            "unique_bias_GBps": round(unique_bias_bytes(w) / (dense_ms * 1e-3) / 1e9, 1),
            # bias elements consumed by the MFMA lanes (every batch item re-reads a shared bias, mostly
            # from L2 / Infinity Cache): NOT an HBM figure
            "bias_consumed_GBps": round(w.pairs * 2 / (dense_ms * 1e-3) / 1e9, 1),
            "hbm_bytes_measured": _profile_field(f"fwd_lowrank_{w.name}_hbm_traffic.txt", "dense_traffic_bytes_per_launch"),
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
            dense_bwd_ms, _ = kernel_ms(dense_bwd)
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
            jit_ms, _ = kernel_ms(jit)
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
                jit_bwd_ms, _ = kernel_ms(jit_bwd)
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
        bwd_ms, _ = kernel_ms(bwd)
        result["backward"] = {"ms": round(bwd_ms, 5),
                              "TFLOPs": round(w.bwd_flops() / (bwd_ms * 1e-3) / 1e12, 2),
                              "pct_of_bf16_mfma_peak": round(100 * w.bwd_flops() / (bwd_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2)}
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

            def f2(t=None):
                t = t or d
                api.fb_lowrank_attn_fwd(t["q"], t["k"], t["v"], t["phi_q"], t["phi_k"], out=t["out"],
                                        lse=t["lse"], causal=w_.causal, stream=stream)

            def d2(t=None):
                t = t or d
                api.fb_dense_bias_attn_fwd(t["q"], t["k"], t["v"], t["bias"], out=t["out"], lse=t["lse"],
                                           causal=w_.causal, stream=stream)
            ms_lr, _ = kernel_ms(f2)
            ms_de, _ = kernel_ms(d2)
            fl = wo.fwd_flops()
            row = {"B": wo.B, "H": wo.H, "N": wo.N, "C": wo.C, "R": wo.R,
                   "fwd_ms": round(ms_lr, 5),
                   "fwd_TFLOPs": round(fl / (ms_lr * 1e-3) / 1e12, 2),
                   "pct_of_bf16_mfma_peak": round(100 * fl / (ms_lr * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2),
                   "dense_ms": round(ms_de, 5),
                   "dense_unique_bias_GBps": round(unique_bias_bytes(wo) / (ms_de * 1e-3) / 1e9, 1),
                   "dense_bias_consumed_GBps": round(wo.pairs * 2 / (ms_de * 1e-3) / 1e9, 1),
                   "speedup_lowrank_vs_dense": round(ms_de / ms_lr, 3)}
            # algorithmic HBM bytes of the low-rank forward: q, k, v, out, the factors, lse
            lr_keys = ("q", "k", "v", "out", "lse", "phi_q", "phi_k")
            alg_bytes = tensor_bytes({k_: d[k_] for k_ in lr_keys})
            if tensor_bytes(d) < (256 << 20):
                # fits the Infinity Cache: back-to-back launches are "hot"; time the cold case as well
                lr_set = {k_: d[k_] for k_ in lr_keys}
                cold_lr, nset, sets = rotating(f2, lr_set, tensor_bytes(lr_set))
                ms_lr_cold, _ = kernel_ms(cold_lr)
                del sets
                de_set = {k_: d[k_] for k_ in ("q", "k", "v", "out", "lse", "bias")}
                cold_de, nset_d, sets = rotating(d2, de_set, tensor_bytes(de_set))
                ms_de_cold, _ = kernel_ms(cold_de)
                del sets
                torch.cuda.empty_cache()
                row.update({"fwd_ms_cold": round(ms_lr_cold, 5), "dense_ms_cold": round(ms_de_cold, 5),
                            "cold_buffer_sets": [nset, nset_d],
                            "speedup_lowrank_vs_dense_cold": round(ms_de_cold / ms_lr_cold, 3)})
            if name == "pairformer":
                cold = row.get("fwd_ms_cold", ms_lr)
                row["roofline"] = {"bound": "hbm", "unit": "GB/s", "peak": PEAK_HBM_GBS,
                                   "algorithmic_bytes": alg_bytes,
                                   "achieved": round(alg_bytes / (cold * 1e-3) / 1e9, 1),
                                   "frac": round(alg_bytes / (cold * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                   "achieved_hot": round(alg_bytes / (ms_lr * 1e-3) / 1e9, 1),
                                   "note": "achieved = algorithmic bytes / cold-cache launch time; hot launches "
                                           "are served from the Infinity Cache"}
            elif name == "vision_relpos":
                sm = wo.pairs * SOFTMAX_FLOP_PER_PAIR
                row["roofline"] = {"bound": "alu", "unit": "TFLOP/s", "peak": PEAK_VALU_TFLOPS,
                                   "achieved": round(sm / (ms_lr * 1e-3) / 1e12, 2),
                                   "frac": round(sm / (ms_lr * 1e-3) / 1e12 / PEAK_VALU_TFLOPS, 4),
                                   "flop_per_pair": SOFTMAX_FLOP_PER_PAIR,
                                   "note": "softmax vector work (multiply-add, exponential at quarter rate, "
                                           "convert, row sum) against the fp32 vector rate without packed ops"}
            else:
                row["roofline"] = {"bound": "mfma", "unit": "TFLOP/s", "peak": PEAK_BF16_TFLOPS,
                                   "achieved": row["fwd_TFLOPs"], "frac": round(row["fwd_TFLOPs"] / PEAK_BF16_TFLOPS, 4)}
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
                    f_ms_db, _ = kernel_ms(db2, steps=3, repeats=3)
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
                ms_b, _ = kernel_ms(b2, steps=5)
                row["bwd_ms"] = round(ms_b, 4)
                row["bwd_TFLOPs"] = round(wo.bwd_flops() / (ms_b * 1e-3) / 1e12, 2)
                row["bwd_pct_of_bf16_mfma_peak"] = round(100 * wo.bwd_flops() / (ms_b * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2)
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
        ms_f, _ = kernel_ms(f3)
        ms_b, _ = kernel_ms(b3)
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
        ms_f5, _ = kernel_ms(f3)
        ms_b5, _ = kernel_ms(b3)
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
        ms_m, _ = kernel_ms(fm_)
        ms_p, _ = kernel_ms(plain)
        dom = torch.randn((Bm, Hm, Nm, Cm), device="cuda", generator=g).to(torch.bfloat16)
        wsb = torch.empty(api.fb_lowrank_mulbias_attn_bwd_workspace_bytes(Bm, Hm, Nm, Cm, 2), dtype=torch.uint8,
                          device="cuda")
        fm_()

        def bm_():
            api.fb_lowrank_mulbias_attn_bwd(qm, km, vm, fm, fm, om, lm, dom, workspace=wsb, stream=stream)
        ms_mb, _ = kernel_ms(bm_)
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
