"""CPU-side checks of the C-ABI library: it loads, and it exports every symbol that
include/first.h declares (no compute calls: there is no GPU here)."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "first.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(first_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound():
    import paper_2410_12513_amd as P
    if not os.path.exists(P.lib_path()):
        from paper_2410_12513_amd.build import build
        build()
    lib = P.load_library()
    names = _declared()
    assert len(names) >= 18
    for n in names:
        assert hasattr(lib, n), f"{n} declared in first.h but not exported"
    assert sorted(P.EXPORTS) == names


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import paper_2410_12513_amd.binding as B
    monkeypatch.setattr(B, "_LIB", None)
    monkeypatch.setattr(B, "HERE", str(tmp_path))
    with pytest.raises(FileNotFoundError):
        B.load_library()


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2410_12513_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("no CPU fallback", ""), f"{f} mentions the oracle"


def test_build_reads_resource_remarks_and_limits_scratch():
    """The build refuses a library in which a kernel that keeps loads in flight through inline asm spills registers."""
    from paper_2410_12513_amd import build as B
    text = """
a.h:10:1: remark: Function Name: _ZN5first6k_stepILi128ELb1EEEvNS_10StepParamsE [-Rpass-analysis=kernel-resource-usage]
a.h:10:1: remark:     VGPRs: 233 [-Rpass-analysis=kernel-resource-usage]
a.h:10:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
a.h:10:1: remark:     VGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]
b.h:20:1: remark: Function Name: _ZN5first8k_gateupINS_4bf16EEEvNS_9DecParamsE [-Rpass-analysis=kernel-resource-usage]
b.h:20:1: remark:     VGPRs: 64 [-Rpass-analysis=kernel-resource-usage]
b.h:20:1: remark:     ScratchSize [bytes/lane]: 288 [-Rpass-analysis=kernel-resource-usage]
b.h:20:1: remark:     VGPRs Spill: 89 [-Rpass-analysis=kernel-resource-usage]
"""
    r = B.kernel_resources(text)
    assert r["_ZN5first6k_stepILi128ELb1EEEvNS_10StepParamsE"] == {"vgprs": 233, "scratch": 0, "spills": 0}
    assert r["_ZN5first8k_gateupINS_4bf16EEEvNS_9DecParamsE"] == {"vgprs": 64, "scratch": 288, "spills": 89}
    assert B.SCRATCH_LIMITS["k_step"] == 0 and B.SCRATCH_LIMITS["k_attn_mfma_b"] == 0
