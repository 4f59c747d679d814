"""CPU-only checks of the library's host side: the C-ABI exports what ``include/reft.h`` declares,
argument validation, and the plan's integer arithmetic (prefix sums, bucket ranges, tile table,
SplitParameter cut) against numpy.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2310_12670_amd as reft
from workload import make_workload, span_nbytes

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "reft.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(reft_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert len(names) >= 20
    lib = ctypes.CDLL(reft.lib_path())
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in reft.h but not exported"
    # and the binding offers the same names
    for n in names:
        assert hasattr(reft, n), f"binding lacks {n}"


@pytest.fixture
def host_only():
    reft.reft_set_tunable("host_only_plans", 1)
    yield
    reft.reft_set_tunable("host_only_plans", 0)


def test_plan_arithmetic_matches_numpy(host_only):
    rng = np.random.default_rng(5)
    for trial in range(20):
        T = int(rng.integers(1, 200))
        sizes = rng.integers(0, 300000, size=T)
        sizes[rng.integers(0, T, size=T // 5)] = 0
        if trial == 0:
            sizes[:] = 0
        L = int(sizes.sum())
        buckets = []
        left = L
        while left:
            n = min(left, 2 * int(rng.integers(1, 1 << 19)) + 1)
            buckets.append(n)
            left -= n
        plan = reft.reft_plan_create(sizes.tolist(), buckets)
        try:
            assert reft.reft_plan_stream_bytes(plan) == L
            assert reft.reft_plan_num_spans(plan) == T
            assert reft.reft_plan_num_buckets(plan) == len(buckets)
            assert reft.reft_plan_max_bucket_bytes(plan) == (max(buckets) if buckets else 0)
            ends = np.cumsum(sizes)
            for t in rng.integers(0, T + 1, size=10):
                want = 0 if t == 0 else int(ends[t - 1])
                assert reft.reft_plan_span_offset(plan, int(t)) == want
            bends = np.cumsum(buckets) if buckets else np.array([], dtype=np.int64)
            for b in range(min(len(buckets), 5)):
                lo, hi = reft.reft_plan_bucket_range(plan, b)
                assert hi == bends[b] and lo == (bends[b - 1] if b else 0)
            tile, ntiles = reft.reft_plan_tile_info(plan)
            assert ntiles == -(-L // tile)
            for t in range(ntiles):
                want = int(np.searchsorted(ends, t * tile, side="right"))
                assert reft.reft_plan_tile_first_span(plan, t) == want
            assert reft.reft_plan_staging_slot_bytes(plan) >= (max(buckets) if buckets else 0) + 256
            for o in [0, L] + [int(x) for x in rng.integers(0, L + 1, size=8)]:
                want_b = int(np.searchsorted(bends, o, side="right")) if len(buckets) else 0
                assert reft.reft_plan_bucket_of(plan, o) == want_b
            with pytest.raises(reft.ReftError):
                reft.reft_plan_bucket_of(plan, L + 1)
        finally:
            reft.reft_plan_destroy(plan)


def test_uniform_buckets(host_only):
    for L, bucket in ((0, 7), (1, 7), (14, 7), (15, 7), (100, 1000)):
        plan = reft.reft_plan_create([L], None, bucket)
        try:
            nb = -(-L // bucket)
            assert reft.reft_plan_num_buckets(plan) == nb
            covered = 0
            for b in range(nb):
                lo, hi = reft.reft_plan_bucket_range(plan, b)
                assert lo == covered and 0 < hi - lo <= bucket
                covered = hi
            assert covered == L
        finally:
            reft.reft_plan_destroy(plan)


def test_split_parameter_cut(host_only):
    """Algorithm 1, SplitParameter: the prefix W[:floor(n t_bubble / t_ss)] and the rest cover
    [0, n) exactly once; a bubble longer than the snapshot takes everything."""
    plan = reft.reft_plan_create([1000, 24, 0, 1])
    try:
        n = 1025
        assert reft.reft_plan_split(plan, 0.0, 1.0) == 0
        assert reft.reft_plan_split(plan, 1.0, 1.0) == n
        assert reft.reft_plan_split(plan, 5.0, 1.0) == n
        assert reft.reft_plan_split(plan, 1.0, 3.0) == n // 3
        assert reft.reft_plan_split(plan, 0.25, 0.5) == n // 2
        for bad in ((1.0, 0.0), (-1.0, 1.0), (1.0, float("nan"))):
            with pytest.raises(reft.ReftError) as e:
                reft.reft_plan_split(plan, *bad)
            assert e.value.code == reft.REFT_EINVAL
    finally:
        reft.reft_plan_destroy(plan)


def test_plan_rejects_bad_arguments(host_only):
    cases = [
        (dict(span_nbytes=[], bucket_nbytes=[]), reft.REFT_EINVAL),          # T == 0
        (dict(span_nbytes=[10], bucket_nbytes=[5, 0, 5]), reft.REFT_EINVAL),  # empty bucket
        (dict(span_nbytes=[10], bucket_nbytes=[5, 4]), reft.REFT_ESIZE),      # short
        (dict(span_nbytes=[10], bucket_nbytes=[5, 6]), reft.REFT_ESIZE),      # long
        (dict(span_nbytes=[10], bucket_nbytes=[]), reft.REFT_ESIZE),          # none
        (dict(span_nbytes=[2 ** 63, 2 ** 63], bucket_nbytes=[1]), reft.REFT_ESIZE),  # overflow
    ]
    for kw, code in cases:
        with pytest.raises(reft.ReftError) as e:
            reft.reft_plan_create(**kw)
        assert e.value.code == code, kw
        assert reft.reft_last_error()


def test_host_only_plan_is_refused_by_gpu_calls(host_only):
    plan = reft.reft_plan_create([16])
    try:
        with pytest.raises(reft.ReftError) as e:
            reft.reft_parity_encode(plan, [1234], 1, 5678)
        assert e.value.code == reft.REFT_EINVAL
    finally:
        reft.reft_plan_destroy(plan)


def test_reconstruct_argument_checks_need_no_gpu():
    """More than one lost shard is beyond one parity (section 4.2): refused, not mis-decoded."""
    with pytest.raises(reft.ReftError) as e:
        reft.reft_reconstruct([None, 4096, None, 8192], 12288, 64, 16384)
    assert e.value.code == reft.REFT_EUNRECOVERABLE
    with pytest.raises(reft.ReftError) as e:
        reft.reft_reconstruct([4096, 8192], 12288, 64, 16384)          # nothing lost
    assert e.value.code == reft.REFT_EINVAL
    with pytest.raises(reft.ReftError) as e:
        reft.reft_reconstruct([None] + [4096] * 31, 12288, 64, 16384)  # k too large
    assert e.value.code == reft.REFT_EINVAL
    with pytest.raises(reft.ReftError) as e:
        reft.reft_reconstruct([None, 4096], None, 64, 16384)           # null parity
    assert e.value.code == reft.REFT_EINVAL


def test_tunables():
    for name, good, bad in (("unroll", 2, 3), ("nontemporal", 0, 2), ("tile_shift", 14, 40),
                            ("max_wgs", 64, 1 << 30), ("link_wgs", 8, 0), ("dma_streams", 2, 3),
                            ("gather_min_pieces", 3, 0), ("graph_copies", 2, 3), ("small_pieces", 5, 1 << 40),
                            ("burst", 0, 2), ("burst_min_rows", 2, 0),
                            ("burst_stage_bytes", 16384, 5000), ("burst_stage_bytes", 65536, 131072),
                            ("burst_wgs_per_cu", 3, 9), ("burst_max_polls", 0, 1 << 20),
                            ("burst_nap", 4, 4096)):
        old = reft.reft_get_tunable(name)
        reft.reft_set_tunable(name, good)
        assert reft.reft_get_tunable(name) == good
        with pytest.raises(reft.ReftError):
            reft.reft_set_tunable(name, bad)
        reft.reft_set_tunable(name, old)
    for name in ("dma_min_bytes", "burst_min_bytes"):        # any value is valid
        old = reft.reft_get_tunable(name)
        reft.reft_set_tunable(name, 12345)
        assert reft.reft_get_tunable(name) == 12345
        reft.reft_set_tunable(name, old)
    with pytest.raises(reft.ReftError):
        reft.reft_set_tunable("no_such_knob", 1)
    with pytest.raises(reft.ReftError):
        reft.reft_get_tunable("no_such_knob")


def test_plans_of_the_five_configurations(host_only):
    """Sizes of the full configurations (spans, buckets, stream bytes)."""
    want = {0: (256, 4, 14680064), 1: (1164, 176, 11795488768), 2: (724, 679, 11391385600),
            3: (436, 224, 14994767872), 4: (364, None, 15434711040)}
    for cfg, (T, NB, L) in want.items():
        wl = make_workload(cfg)
        plan = reft.reft_plan_create(span_nbytes(wl), wl.bucket_nbytes)
        try:
            assert reft.reft_plan_num_spans(plan) == T
            assert reft.reft_plan_stream_bytes(plan) == L == wl.L
            if NB is not None:
                assert reft.reft_plan_num_buckets(plan) == NB
            else:
                assert all(b % 2 == 1 for b in wl.bucket_nbytes[:-1])
                assert all((1 << 20) <= b <= (1 << 27) for b in wl.bucket_nbytes[:-1])
        finally:
            reft.reft_plan_destroy(plan)


def test_build_refuses_burst_kernels_that_need_too_many_registers():
    """Two 5-wave workgroups of a burst kernel fit on a compute unit only up to 128 vector
    registers per lane; the build reads the compiler's resource remarks and fails beyond that."""
    from paper_2310_12670_amd.build import check_burst_registers

    def remarks(name, vgprs):
        return (f"x.hip:1:1: remark: Function Name: {name} [-Rpass-analysis=kernel-resource-usage]\n"
                f"x.hip:1:1: remark:     SGPRs: 100 [-Rpass-analysis=kernel-resource-usage]\n"
                f"x.hip:1:1: remark:     VGPRs: {vgprs} [-Rpass-analysis=kernel-resource-usage]\n")

    ok = remarks("_ZN4reft14k_gather_burstILi8ELi4ELb1EEEvX", 121) + remarks("_ZN4reft8k_gatherILi8ELi4ELb1EEEvX", 167)
    assert check_burst_registers(ok) == {"_ZN4reft14k_gather_burstILi8ELi4ELb1EEEvX": 121}
    with pytest.raises(RuntimeError):
        check_burst_registers(ok + remarks("_ZN4reft18k_xor_contig_burstILi8ELi4ELb1EEEvX", 129))
    with pytest.raises(RuntimeError):
        check_burst_registers(remarks("_ZN4reft8k_gatherILi8ELi4ELb1EEEvX", 167))   # no burst kernel reported


def test_header_is_plain_c(tmp_path):
    """include/reft.h is the boundary: it must compile as C99 and as C++ with no other header of
    the project."""
    import shutil
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "t.c"
    src.write_text('#include "reft.h"\nint main(void) { return reft_version() == 0; }\n')
    inc = os.path.join(root, "include")
    if shutil.which("gcc"):
        subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                        "-I", inc, str(src)], check=True)
    if shutil.which("g++"):
        subprocess.run(["g++", "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++",
                        "-I", inc, str(src)], check=True)
