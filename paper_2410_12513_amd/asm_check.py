"""Static check of this library's own device code: destinations of loads that are kept in flight.

Several kernels issue global loads through inline asm and wait for them by count (`s_waitcnt vmcnt(N)`), so that
loads stay in flight across barriers and other work.  The compiler believes such a destination register holds its
value from the asm statement on.  If it lets go of the register before the wait that covers the load (because the
value is dead, or spilled, or copied), whatever it puts there next is overwritten when the load lands - an address,
in the case that was seen, and the kernel faults.  This module compiles the library's source to assembly and walks
every kernel whose name contains one of the given keys: a register written by a global load is "in flight" until a
vmcnt wait covers it (loads return in order: `vmcnt(N)` leaves the N youngest outstanding), and no other instruction
may name it before that.  A straight-line scan, so a heuristic - but it is exactly the pattern of the fault it guards
against.  Needs hipcc only, no GPU."""
from __future__ import annotations

import os
import re
import subprocess
import tempfile

from .build import FLAGS, SRC

KERNELS = ("k_step", "k_attn_tiles_b", "k_attn_mfma_b", "k_bgemv", "k_gemm_nt_bf16_hl")


def _regs(tok: str):
    m = re.match(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return list(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return [int(m.group(1))] if m else []


def assembly() -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in FLAGS if f not in ("-fPIC", "-shared", "-Rpass-analysis=kernel-resource-usage")]
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "first.s")
        res = subprocess.run([hipcc] + flags + ["-S", "--cuda-device-only", SRC, "-o", out], capture_output=True, text=True, cwd=tmp)
        if res.returncode != 0:
            raise RuntimeError("hipcc -S failed:\n" + res.stderr[-2000:])
        with open(out) as fh:
            return fh.read()


def touched_in_flight(asm: str, keys=KERNELS):
    """[(kernel, line number, instruction, registers)] for every instruction that names a load destination in flight."""
    found, fn, inflight = [], None, {}
    for n, line in enumerate(asm.split("\n")):
        if re.match(r"^_Z\S+:$", line):
            fn, inflight = line[:-1], {}
            continue
        t = line.strip()
        if fn is None or not any(k in fn for k in keys) or not t or t[0] in ";.":
            continue
        if t.startswith("global_load_"):
            for r in _regs(t.split()[1].rstrip(",")):
                inflight[r] = n
            continue
        m = re.match(r"s_waitcnt.*vmcnt\((\d+)\)", t)
        if m:
            k, issued = int(m.group(1)), sorted(set(inflight.values()))
            keep = set(issued[len(issued) - k:]) if k > 0 else set()
            inflight = {r: ln for r, ln in inflight.items() if ln in keep}
            continue
        used = set()
        for tok in re.findall(r"v\[\d+:\d+\]|v\d+", t):
            used.update(_regs(tok))
        bad = sorted(r for r in used if r in inflight)
        if bad:
            found.append((fn, n, t, bad))
    return found


if __name__ == "__main__":
    hits = touched_in_flight(assembly())
    for h in hits[:20]:
        print(h)
    print("instructions that touch a load destination in flight:", len(hits))
