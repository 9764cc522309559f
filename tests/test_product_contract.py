"""Contracts of the product path that need no GPU: no CPU fallback, one GPU only, and no import of the oracle."""
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_missing_library_raises_instead_of_falling_back(monkeypatch, tmp_path):
    from paper_2602_03495_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB", str(tmp_path / "no_such_library.so"))
    with pytest.raises(binding.MoeError, match="missing"):
        binding.load_library()


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120, cwd=ROOT)
    assert r.returncode == 2
    assert "one GPU only" in r.stderr
    assert r.stdout.strip() == ""


def test_package_never_imports_the_oracle():
    # the oracle is test infrastructure: only tests/, smoke() and the cpu_baseline leg of bench.py may touch it
    pkg = os.path.join(ROOT, "paper_2602_03495_amd")
    pat = re.compile(r"^\s*(import\s+oracle|from\s+oracle\b)", re.M)
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f), errors="replace").read()
                assert not pat.search(text), f
                assert "oracle/" not in text and "moe_oracle" not in text, f
    bench = open(os.path.join(ROOT, "bench.py")).read()
    assert len(pat.findall(bench)) == 1          # the cpu_baseline leg
    # and the oracle shares nothing with the product: no include of the library's headers, no import of the package
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f), errors="replace").read()
            assert "paper_2602_03495_amd" not in text and "moe_layer.h" not in text and "moe_common.h" not in text, f
