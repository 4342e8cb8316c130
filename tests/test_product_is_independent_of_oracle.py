"""The product path (package, bench's GPU legs) never touches the oracle, and fails loudly
when the HIP library is missing instead of falling back to anything on the CPU."""
import os
import re

import pytest

from paper_2601_16238_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_package_sources_do_not_mention_the_oracle():
    pkg = os.path.join(ROOT, "paper_2601_16238_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), f
                assert "attn_oracle" not in text and "rowops_oracle" not in text, f


def test_oracle_sources_do_not_use_the_product():
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            # no import of the package, no include of its headers, no HIP runtime
            assert "paper_2601_16238_amd" not in text, f
            assert not re.search(r"#\s*include\s*[<\"](?!math|stdint|stdlib|string|omp)", text), f
            assert "hip_runtime" not in text and "libmi355attn" not in text, f


def test_missing_library_raises_instead_of_falling_back(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libmi355attn.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.lib()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "single-GPU" in r.stderr
