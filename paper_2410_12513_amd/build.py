"""Builds libfirst.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "first_api.hip")
LIB = os.path.join(HERE, "libfirst.so")

# -packed-fp32-ops is switched off for all device code of this library.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Rpass-analysis=kernel-resource-usage"]

# Register spills are a correctness matter for the kernels that keep loads in flight through inline asm (the exchange
# polls of the persistent step kernel, the attention kernels of the batched path, the partial sums a last arriver
# collects, the operand prefetch of the prefill GEMM): the compiler does not know that the destination of such a load is
# written later, so a destination it spills and hands to another value is overwritten when the load lands.  Bytes of
# scratch per lane each kernel may use (k_attn_tiles_b: a handful of loop-invariant values the compiler parks there under
# the kernel's 128-register cap; asm_check.py verifies that no in-flight destination is among them, or is touched in any
# other way; "k_bgemv" covers k_bgemv and k_bgemv_g):
SCRATCH_LIMITS = {"k_step": 0, "k_attn_tiles_b": 32, "k_attn_mfma_b": 0, "k_bgemv": 0, "k_gemm_nt_bf16_hl": 0}


def kernel_resources(remarks: str) -> dict:
    """{mangled kernel name: {"vgprs": n, "scratch": bytes per lane, "spills": n}} from hipcc's resource-usage remarks."""
    out, name = {}, None
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            out[name] = {}
            continue
        if name is None:
            continue
        for key, pat in (("vgprs", r" VGPRs: (\d+)"), ("scratch", r"ScratchSize \[bytes/lane\]: (\d+)"),
                         ("spills", r"VGPRs Spill: (\d+)")):
            m = re.search(pat, line)
            if m:
                out[name][key] = int(m.group(1))
    return out


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + [SRC, "-o", LIB + ".tmp"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    kept, skip = [], 0
    for l in res.stderr.splitlines():                  # drop the resource remarks (each followed by a source line and a caret line)
        if "kernel-resource-usage" in l:
            skip = 2
        elif skip and re.match(r"\s+(\d+ )?\|", l):
            skip -= 1
        elif "packed-fp32-ops" not in l and not l.startswith("In file included from"):
            skip = 0
            kept.append(l)
    err = "\n".join(kept)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    for kernel, use in kernel_resources(res.stderr).items():
        for key, limit in SCRATCH_LIMITS.items():
            if key in kernel and use.get("scratch", 0) > limit:
                os.remove(LIB + ".tmp")
                raise RuntimeError(f"{kernel}: {use['scratch']} bytes of scratch per lane ({use.get('spills', '?')} spilled registers), "
                                   f"limit {limit}: this kernel keeps loads in flight in registers and must not spill them")
    if verbose and err.strip():
        sys.stderr.write(err + "\n")
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
