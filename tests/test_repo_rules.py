"""Structural rules of the repository, checked on the CPU: the product never touches the oracle,
the oracle never touches the product, and bench.py refuses more than one GPU."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _sources(*dirs, exts=(".py", ".hip", ".hpp", ".h", ".c")):
    for d in dirs:
        for base, _, files in os.walk(os.path.join(ROOT, d)):
            if "__pycache__" in base:
                continue
            for f in files:
                if f.endswith(exts):
                    yield os.path.join(base, f)


def test_product_does_not_use_the_oracle_and_vice_versa():
    for path in _sources("paper_2310_12670_amd", "include"):
        text = open(path).read()
        assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), path
        assert "reft_oracle" not in text and "libreft_oracle" not in text, path
    for path in _sources("oracle"):
        text = open(path).read()
        assert "paper_2310_12670_amd" not in text and "libreft.so" not in text, path
        assert not re.search(r"#include\s+\"(\.\./)*(include|paper_2310_12670_amd)", text), path
    # the input generator holds none of the method's arithmetic
    for path in _sources("workload"):
        text = open(path).read()
        assert "oracle" not in re.sub(r'""".*?"""', "", text, flags=re.S), path
        assert "bitwise_xor" not in text and "paper_2310_12670_amd" not in text, path


def test_bench_uses_the_oracle_only_for_the_cpu_baseline():
    text = open(os.path.join(ROOT, "bench.py")).read()
    uses = [m.start() for m in re.finditer(r"^\s*import oracle\b", text, re.M)]
    assert len(uses) == 1
    start = text.index("def cpu_baseline(")
    nxt = text.index("\nif __name__", start)
    assert start < uses[0] < nxt


def test_nothing_committed_reads_the_working_folder_or_the_reference():
    for path in list(_sources("paper_2310_12670_amd", "oracle", "workload", "include")) + \
            [os.path.join(ROOT, "bench.py"), os.path.join(ROOT, "__graft_entry__.py")]:
        text = open(path).read()
        assert not re.search(r"(^|[\"'/\s(])_work(/|[\"'])", text, re.M), path
        assert "/root/reference" not in text, path


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr
