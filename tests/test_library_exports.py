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
