"""Builds libflashbias.so (HIP kernels + C-ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libflashbias.so")
PROBE_LIB = os.path.join(HERE, "libfb_bench_probe.so")     # bench-only probes, never linked into the product

SOURCES = ["fb_api.hip", "fb_fwd_f32.hip", "fb_fwd_bf16.hip", "fb_fwd_bf16_c16.hip", "fb_fwd_bf16_c32.hip",
           "fb_fwd_bf16_c64.hip", "fb_fwd_bf16_c128.hip", "fb_fwd_bf16_alibi.hip", "fb_bwd_bf16.hip", "fb_bwd_f32.hip",
           "fb_mulbias.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-ffast-math", "-fno-finite-math-only",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    srcp = os.path.join(CSRC, src)
    deps = [srcp] + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    deps.append(os.path.join(HERE, "..", "include", "flashbias.h"))
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps):
        return obj
    extra = os.environ.get("FB_EXTRA_FLAGS", "").split()
    cmd = [_hipcc(), *FLAGS, *extra, "-c", srcp, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError(f"hipcc failed on {src}")
    errs = "\n".join(l for l in r.stderr.splitlines()
                     if "packed-fp32-ops" not in l and l.strip())
    # the direct-to-LDS loads name m0 as clobbered on purpose; clang notes that it is a reserved register
    if "Reserved registers on the clobber list" in errs or "inline asm clobber list contains reserved registers" in errs:
        errs = ""
    if errs:
        sys.stderr.write(errs + "\n")
    return obj


def build(force: bool = True, jobs: int = 7) -> str:
    """Compile every kernel source and link the shared library.  force=False reuses objects
    that are newer than all sources and headers."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    # only the C-ABI leaves the library: kernel stubs and helpers with external linkage stay local
    vers = os.path.join(OBJ, "exports.map")
    with open(vers, "w") as f:
        f.write("{ global: fb_*; local: *; };\n")
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", f"-Wl,--version-script={vers}", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("link failed")
    # the bench-only probe library (MFMA-loop ceiling, calibration copy)
    pobj = _compile("fb_bench_probe.hip", force)
    pvers = os.path.join(OBJ, "probe_exports.map")
    with open(pvers, "w") as f:
        f.write("{ global: fbp_*; local: *; };\n")
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", f"-Wl,--version-script={pvers}", "-o", PROBE_LIB, pobj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("probe link failed")
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))
