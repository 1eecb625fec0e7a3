"""Build-time check for the hand-placed MFMA forms (csrc/fb_device.h: mfma32_vdst*).

An MFMA written as inline assembly is opaque to the compiler, which therefore inserts none of the
wait states its result needs before another kind of instruction may read or overwrite it (11 after
an 8-pass MFMA on gfx950).  The kernels keep that distance by construction at the end of every
chain; what the register allocator does between the links of a chain cannot be constrained from
the source.  This script compiles a kernel source to assembly with the library's flags and scans
every kernel: after each MFMA with a VGPR result, no instruction other than the next link of the
same chain may touch the result registers within the window (`s_nop N` counts N + 1 wait states,
any other instruction one; the scan of a result ends at a branch, where the source-level fence has
already been issued for chain ends).  Compiler-placed MFMAs pass trivially (the compiler pads them).

    python -m paper_2505_12044_amd.check_mfma_hazards            # exits 1 when a candidate is found
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

from . import build as fb_build

WINDOW = 11
SOURCES = ["fb_bwd_bf16.hip"]       # the sources that use the hand-placed forms


def _regs(tok: str) -> set:
    tok = tok.strip()
    m = re.match(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)\b", tok)
    return {int(m.group(1))} if m else set()


def scan_asm(text: str, window: int = WINDOW):
    """Returns (number of VGPR-result MFMAs seen, list of (kernel, mfma, offender) candidates)."""
    found, seen = [], 0
    kern, ins = None, []

    def scan(kern, ins):
        nonlocal seen
        for i, line in enumerate(ins):
            if not line.startswith("v_mfma"):
                continue
            ops = [t.strip() for t in line.split(None, 1)[1].split(",")]
            dst = _regs(ops[0])
            if not dst:
                continue                      # AGPR result: a compiler-placed form
            seen += 1
            ws = 0
            for x in ins[i + 1:]:
                if ws >= window:
                    break
                if x.startswith("s_nop"):
                    ws += int(x.split()[1]) + 1
                    continue
                toks = (x.split(None, 1)[1] if " " in x else "").split(",")
                touched = set()
                for t in toks:
                    for piece in re.findall(r"v\[\d+:\d+\]|v\d+\b", t):
                        touched |= _regs(piece)
                if x.startswith("v_mfma"):
                    xdst = _regs(toks[0]) if toks else set()
                    if xdst == dst:
                        break                 # the next link of the same chain
                    if touched & dst:
                        found.append((kern, line, x))
                elif touched & dst:
                    found.append((kern, line, x))
                if x.startswith(("s_cbranch", "s_branch", "s_endpgm")):
                    break
                ws += 1

    for raw in text.split("\n"):
        c = raw.split(";")[0].rstrip()
        if re.match(r"^_Z\w+:", c):
            if kern:
                scan(kern, ins)
            kern, ins = c[:-1], []
            continue
        t = c.strip()
        if not t or t.startswith(".") or t.endswith(":"):
            continue
        ins.append(t)
    if kern:
        scan(kern, ins)
    return seen, found


def check(sources=SOURCES):
    total_seen, total_found = 0, []
    with tempfile.TemporaryDirectory() as tmp:
        for src in sources:
            out = os.path.join(tmp, src.replace(".hip", ".s"))
            cmd = [fb_build._hipcc(), *fb_build.FLAGS, "-S", "--cuda-device-only",
                   os.path.join(fb_build.CSRC, src), "-o", out]
            r = subprocess.run(cmd, capture_output=True, text=True)
            if r.returncode != 0:
                sys.stderr.write(r.stdout + r.stderr)
                raise RuntimeError(f"hipcc failed on {src}")
            seen, found = scan_asm(open(out).read())
            total_seen += seen
            total_found += found
    return total_seen, total_found


if __name__ == "__main__":
    seen, found = check()
    for kern, mfma, x in found:
        print(f"{kern}: {mfma}  ->  {x}")
    print(f"VGPR-result MFMAs scanned: {seen}; hazard candidates: {len(found)}")
    sys.exit(1 if found else 0)
