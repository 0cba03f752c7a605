"""bench.py's command line on a box without a GPU: what it refuses, and that nothing of the product imports the oracle."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "--gpus 1" in r.stderr and "one MI355X" in r.stderr
    assert not r.stdout.strip()  # no JSON line that could be taken for a measurement


def test_the_package_never_imports_the_oracle_or_working_files():
    pkg = os.path.join(ROOT, "paper_2605_06914_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".h", ".hip")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), f
                assert not re.search(r"(?<![A-Za-z0-9])_work(?![A-Za-z0-9_])", text), f
    for f in ("bench.py", "__graft_entry__.py"):
        assert not re.search(r"(?<![A-Za-z0-9])_work(?![A-Za-z0-9_])", open(os.path.join(ROOT, f)).read()), f
