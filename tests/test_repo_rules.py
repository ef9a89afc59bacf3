"""Checks of the repository's own rules that need no GPU: the product package never touches the
oracle, bench.py refuses more than one GPU, and the header, binding and library agree on names."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2210_08803_amd")


def test_product_package_never_uses_the_oracle():
    for dirpath, _, files in os.walk(PKG):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f), encoding="utf-8").read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), f
                assert "liboracle" not in text and "oracle.cpp" not in text, f


def test_oracle_never_uses_the_product_package():
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".cpp")):
            text = open(os.path.join(ROOT, "oracle", f), encoding="utf-8").read()
            assert "paper_2210_08803_amd" not in text and "libhctr" not in text and "hctr.h" not in text, f


def test_bench_refuses_more_than_one_gpu():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""
