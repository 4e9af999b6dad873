"""Structure rules that the parity claims rest on, checked on the sources (no GPU):
the product never reaches the oracle, the oracle never reaches the product, and the
benchmark refuses more than one GPU before it touches any."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2408_16978_amd")
ORACLE = os.path.join(ROOT, "oracle")


def _sources(top, exts):
    for d, _, files in os.walk(top):
        if os.path.basename(d) in ("_build", "__pycache__"):
            continue
        for f in files:
            if f.endswith(exts):
                yield os.path.join(d, f)


def test_product_never_imports_or_links_the_oracle():
    pat = re.compile(r"^\s*(from|import)\s+oracle\b|libfpdt_oracle|oracle/", re.M)
    for path in _sources(PKG, (".py", ".hip", ".h")):
        assert not pat.search(open(path).read()), path


def test_oracle_never_imports_the_product_or_its_headers():
    pat = re.compile(r"paper_2408_16978_amd|libfpdt\.so|libfpdt_tokenwise|include/fpdt|hip/hip_runtime|\btorch\b")
    for path in _sources(ORACLE, (".py", ".c", ".h")):
        assert not pat.search(open(path).read()), path


def test_oracle_users_are_only_tests_smoke_and_the_cpu_baseline():
    pat = re.compile(r"^\s*(from|import)\s+oracle\b", re.M)
    users = set()
    tracked = [os.path.join(ROOT, f) for f in ("bench.py", "__graft_entry__.py")]
    tracked += list(_sources(PKG, (".py",))) + list(_sources(os.path.join(ROOT, "tests"), (".py",)))
    for path in tracked:
        rel = os.path.relpath(path, ROOT)
        if pat.search(open(path).read()):
            users.add(rel.split(os.sep)[0] if os.sep in rel else rel)
    assert users <= {"tests", "bench.py", "__graft_entry__.py"}, users
    # in bench.py the import sits inside cpu_baseline(), in __graft_entry__.py inside build() / smoke()
    bench = open(os.path.join(ROOT, "bench.py")).read()
    assert bench.count("from oracle") == 1
    assert bench.index("def cpu_baseline") < bench.index("from oracle") < bench.index("def main")


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
