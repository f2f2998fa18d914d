"""The C-ABI library loads on a CPU-only machine and exports every symbol the
header declares (no compute calls here)."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "swiftkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(swiftkv_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    from paper_2410_03960_amd import binding as B
    if not os.path.exists(B.LIB_PATH):
        from paper_2410_03960_amd import build
        build.build(verbose=False)
    lib = B.load()
    names = _declared()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), f"{n} declared in swiftkv.h but not exported"
    assert set(B.EXPORTS) == set(names)
    assert b"gfx950" in lib.swiftkv_version()


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2410_03960_amd import binding as B
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        B.load()


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2410_03960_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("no CPU fallback", ""), f
    osrc = open(os.path.join(ROOT, "oracle", "swiftkv_oracle.py")).read()
    assert "paper_2410_03960_amd" not in osrc and "workloads" not in osrc
