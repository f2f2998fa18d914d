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


def test_bench_refuses_more_than_one_gpu():
    """This build is single-GPU: bench.py --gpus N (N > 1) must say so and exit
    non-zero before touching a GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_workloads_beyond_the_five_configurations_are_consistent():
    """The prompt-chunk and decode-step workloads: batch geometry (cached
    context per sequence, block tables with room for context + new tokens)."""
    import workloads as WL
    wl = WL.get_workload("8b_l16_b8x2048_ctx6144")
    b = WL.build_batch(wl)
    assert b.seq_lens.tolist() == [2048] * 8 and b.context_lens.tolist() == [6144] * 8
    assert b.block_tables.shape[1] == (6144 + 2048) // 16 and b.n_blocks >= 8 * 512
    wl = WL.get_workload("8b_l16_dec64_ctx2048")
    b = WL.build_batch(wl)
    assert b.seq_lens.tolist() == [1] * 64 and b.context_lens.tolist() == [2048] * 64
    assert b.block_tables.shape[1] == 129
    used = b.block_tables.flatten().tolist()
    assert len(set(used)) == len(used)          # no block shared between sequences


def test_header_is_plain_c(tmp_path):
    """include/swiftkv.h is a C header (plain pointers and sizes, no C++ or HIP
    types): a C11 translation unit that includes it and takes the address of
    every declared function must compile with gcc."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    names = _declared()
    src = tmp_path / "use_header.c"
    src.write_text('#include "swiftkv.h"\n'
                   + "const void *const table[] = {" + ", ".join(f"(const void *){n}" for n in names) + "};\n"
                   + "int n_entries(void) { return (int)(sizeof(table) / sizeof(table[0])); }\n")
    r = subprocess.run(["gcc", "-std=c11", "-Wall", "-Werror", "-pedantic", "-Wno-pedantic", "-I", os.path.join(ROOT, "include"),
                        "-c", str(src), "-o", str(tmp_path / "use_header.o")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
