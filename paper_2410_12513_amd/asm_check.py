"""Static check of this library's own device code: destinations of loads that are kept in flight.

Several kernels issue global loads through inline asm and wait for them by count (`s_waitcnt vmcnt(N)`), so that
loads stay in flight across barriers and other work.  The compiler believes such a destination register holds its
value from the asm statement on.  If it touches the register before the wait that covers the load - because the value
is dead, or spilled, or MOVED TO ANOTHER REGISTER (live-range splitting at a branch does that) - it reads or overwrites
something that is not there yet; one such copy gave wrong attention results on the first decode step of a sequence, when
memory is slow, and a reused register once ended in a memory fault.  This module compiles the library's source to
assembly and walks every kernel whose name contains one of the given keys.  Loads inside an inline asm statement (hipcc
brackets those with ;;#ASMSTART / ;;#ASMEND) are "in flight" until a vmcnt wait covers them - every vector memory
operation counts, in issue order: `vmcnt(N)` leaves the N youngest outstanding - and no instruction may name their
destination before that.  Loads the compiler issues itself are its own business.  The walk follows the text and carries
what is in flight along branches (see touched_in_flight); it knows nothing of which path is taken, so it is a heuristic -
but it is exactly the pattern of the faults it guards against.  Needs hipcc only, no GPU."""
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


def _functions(asm: str, keys):
    """[(mangled name, [(line number, stripped instruction or label)])] for the kernels whose name contains a key."""
    out, fn, body = [], None, []
    for n, line in enumerate(asm.split("\n")):
        m = re.match(r"^(_Z\w+):", line)                # (hipcc puts a comment behind the label)
        if m:
            if fn is not None:
                out.append((fn, body))
            fn, body = (m.group(1), []) if any(k in m.group(1) for k in keys) else (None, [])
            continue
        t = line.strip()
        if fn is not None and t.startswith(";;#ASM"):
            body.append((n, t))                          # ;;#ASMSTART / ;;#ASMEND bracket the text of an inline asm statement
            continue
        t = t.split(";")[0].strip()                      # (comments behind instructions and labels)
        if fn is None or not t or (t[0] == "." and not re.match(r"^\.L\S+:$", t)):
            continue
        body.append((n, t))
    if fn is not None:
        out.append((fn, body))
    return out


def touched_in_flight(asm: str, keys=KERNELS):
    """[(kernel, line number, instruction, registers)] for every instruction that names a load destination in flight.

    The walk follows the text of a kernel; what is in flight at a branch is also carried to the branch's target, and
    the walk is repeated until nothing new arrives at any label, so a destination that is requested at the tail of a
    loop and named at its head (or after a forward jump over its wait) is seen as well.  Loads are ordered by the moment
    the walk met them, so what a back edge carries counts as older than what the next trip requests."""
    found = {}
    for fn, body in _functions(asm, keys):
        at_label = {}                                    # label -> {register: sequence number of its load}
        seq = 0
        for _ in range(8):
            grew = False
            inflight, fall = {}, True
            events = []                                  # sequence numbers of the vector memory operations not yet waited for
            in_asm = False
            for n, t in body:
                if t.startswith(";;#ASM"):
                    in_asm = t.startswith(";;#ASMSTART")
                    continue
                m = re.match(r"^(\.L\S+):$", t)
                if m:
                    carried = at_label.get(m.group(1), {})
                    inflight = {**carried, **inflight} if fall else dict(carried)
                    if not fall:
                        events = []
                    events = sorted(set(events) | set(inflight.values()))
                    fall = True
                    continue
                if not fall:
                    continue                             # (unreachable by fall-through, no label yet)
                m = re.match(r"s_c?branch\S*\s+(\.L\S+)", t)
                if m:
                    tgt = at_label.setdefault(m.group(1), {})
                    for r, q in inflight.items():
                        if r not in tgt:
                            tgt[r] = q
                            grew = True
                    if t.startswith("s_branch"):
                        fall = False
                    continue
                m = re.match(r"(global|buffer|scratch|flat)_(load|store|atomic)\w*\s+(\S+)", t)
                if m:                                    # every vector memory operation counts in vmcnt, in issue order
                    seq += 1
                    events.append(seq)
                    returns = m.group(2) == "load" or (m.group(2) == "atomic" and m.group(3).rstrip(",").startswith("v") and
                                                       (" sc0" in t or " glc" in t))
                    if returns and in_asm:               # (the compiler waits for the loads it issues itself before it reuses their registers)
                        for r in _regs(m.group(3).rstrip(",")):
                            inflight[r] = seq
                    continue
                m = re.match(r"s_waitcnt.*vmcnt\((\d+)\)", t)
                if m:
                    k = int(m.group(1))
                    events = events[len(events) - k:] if k > 0 else []
                    keep = set(events)
                    inflight = {r: q for r, q in inflight.items() if q in keep}
                    continue
                used = set()
                for tok in re.findall(r"v\[\d+:\d+\]|v\d+", t):
                    used.update(_regs(tok))
                bad = sorted(r for r in used if r in inflight)
                if bad:
                    found[(fn, n)] = (fn, n, t, bad)
            if not grew:
                break
    return [found[k] for k in sorted(found)]


def kernels_seen(asm: str, keys=KERNELS):
    """{key: number of kernels the walk covers}: a key without kernels means the walk is blind to them."""
    names = [fn for fn, _ in _functions(asm, keys)]
    return {k: sum(k in fn for fn in names) for k in keys}


if __name__ == "__main__":
    hits = touched_in_flight(assembly())
    for h in hits[:20]:
        print(h)
    print("instructions that touch a load destination in flight:", len(hits))
