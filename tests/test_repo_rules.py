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


def test_only_the_diagnostic_call_waits_for_the_whole_device():
    """Data-moving entry points neither wait for the whole device nor allocate device or pinned
    memory: hipDeviceSynchronize appears in reft_plan_burst_stats only, and the allocating calls
    are confined to plan / checkpoint creation and the set-up of derived tables."""
    text = open(os.path.join(ROOT, "paper_2310_12670_amd", "csrc", "reft_api.hip")).read()
    # function bodies by name: text between one top-level definition and the next
    starts = [(m.start(), m.group(1)) for m in re.finditer(
        r"^(?:extern \"C\" |static |template <[^>]*>\nstatic )[^\n;{]*?\b(\w+)\([^;{]*\)\n\{", text, re.M)]
    bodies = {}
    for (a, name), (b, _) in zip(starts, starts[1:] + [(len(text), "")]):
        bodies.setdefault(name, "")
        bodies[name] += text[a:b]
    assert "reft_snapshot_pack_range" in bodies and "upload_ptrs" in bodies and "xor_rows" in bodies
    sync_in = sorted(n for n, b in bodies.items() if "hipDeviceSynchronize" in b)
    assert sync_in == ["reft_plan_burst_stats"], sync_in
    alloc_in = sorted(n for n, b in bodies.items()
                      if re.search(r"\bhip(Malloc|HostMalloc|ExtMallocWithFlags|MallocAsync)\(", b))
    assert alloc_in == ["ensure_zeros", "reft_ckpt_create", "reft_plan_create"], alloc_in
    assert "hipMalloc" not in open(os.path.join(ROOT, "paper_2310_12670_amd", "csrc",
                                                "reft_kernels.hip")).read()
