"""Contracts of the repository layout that need no GPU: the product package and
the CPU oracle stay independent of each other, and bench.py refuses more than
one GPU."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def sources(folder, exts):
    for base, _, files in os.walk(os.path.join(ROOT, folder)):
        for f in files:
            if f.endswith(exts):
                yield os.path.join(base, f)


def test_product_and_oracle_do_not_reference_each_other():
    for path in sources("paper_2004_02297_amd", (".py", ".hip", ".h", ".cpp")):
        text = open(path).read()
        assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), path
        assert "adt_oracle" not in text and "liboracle" not in text, path
    for path in sources("oracle", (".py", ".c", ".h")):
        text = open(path).read()
        assert "paper_2004_02297_amd" not in text and "libadt" not in text, path
        assert '#include "adt' not in text, path
    shared = open(os.path.join(ROOT, "workloads.py")).read()
    assert not re.search(r"^\s*(import|from)\s+(oracle|paper_2004_02297_amd)\b", shared, flags=re.M)


def test_nothing_committed_depends_on_working_files():
    """Working files (probes, sweep scripts, notes) live in an ignored folder; nothing
    that is part of the repository may import, read or run anything there."""
    tracked = subprocess.run(["git", "ls-files"], cwd=ROOT, capture_output=True, text=True, timeout=60)
    if tracked.returncode != 0:
        import pytest
        pytest.skip("not a git checkout")
    for rel in tracked.stdout.split():
        if not rel.endswith((".py", ".h", ".hip", ".c", ".cpp", ".sh")) or rel == "tests/test_repo_contract.py":
            continue
        text = open(os.path.join(ROOT, rel), errors="replace").read()
        assert "_work/" not in text and "_work\"" not in text, rel


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
