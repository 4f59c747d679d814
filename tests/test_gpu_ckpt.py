"""GPU tests of the scheduling units around the snapshot: bucket ranges (what a scheduler places in
a bubble or beside compute, Algorithm 1) and the completed / ongoing snapshot pair (section 4.4).
Expected bytes come from the CPU oracle."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2310_12670_amd as reft
from workload import fill_shard, make_workload, span_nbytes

pytestmark = pytest.mark.gpu
CANARY = 0x5A


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the GPU"
    d = torch.device("cuda:0")
    torch.cuda.set_device(d)
    return d


def host_view(addr, n):
    return np.ctypeslib.as_array((ctypes.c_uint8 * n).from_address(addr))


def setup(dev, bucket=600001, shrink=2):
    wl = make_workload(0, shrink=shrink)
    sizes = span_nbytes(wl)
    plan = reft.reft_plan_create(sizes, None, bucket)
    slot = reft.reft_plan_staging_slot_bytes(plan)
    staging = torch.empty(4 * slot, dtype=torch.uint8, device=dev)
    return wl, sizes, plan, staging


def test_bucket_ranges_compose_in_any_order(dev):
    wl, sizes, plan, staging = setup(dev)
    try:
        L, nb = wl.L, reft.reft_plan_num_buckets(plan)
        assert nb >= 5
        shard = fill_shard(wl, 0, dev)
        want = oracle.pack([oracle.as_bytes(t.cpu()) for t in shard])
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        host = torch.full((L + 64,), CANARY, dtype=torch.uint8, pin_memory=True)
        # a middle range only: everything outside it stays untouched
        reft.reft_snapshot_pack_range(plan, shard, staging, host, 2, 4, s1, s2, host_cap=L)
        reft.reft_snapshot_wait(plan)
        lo, _ = reft.reft_plan_bucket_range(plan, 2)
        _, hi = reft.reft_plan_bucket_range(plan, 3)
        h = host.numpy()
        assert np.array_equal(h[lo:hi], want[lo:hi])
        assert np.all(h[:lo] == CANARY) and np.all(h[hi:] == CANARY)
        # the rest, out of order and with both transports
        reft.reft_snapshot_pack_range(plan, shard, None, host, 4, nb, s1, None, host_cap=L)
        reft.reft_snapshot_pack_range(plan, shard, staging, host, 0, 2, s1, s2, host_cap=L)
        reft.reft_snapshot_pack_range(plan, shard, staging, host, 3, 3, s1, s2, host_cap=L)   # empty
        reft.reft_snapshot_wait(plan)
        torch.cuda.synchronize()
        assert np.array_equal(h[:L], want)
        assert np.all(h[L:] == CANARY)
        with pytest.raises(reft.ReftError) as e:
            reft.reft_snapshot_pack_range(plan, shard, staging, host, 1, nb + 1, s1, s2, host_cap=L)
        assert e.value.code == reft.REFT_EINVAL
    finally:
        reft.reft_plan_destroy(plan)


@pytest.mark.parametrize("t_bubble,t_ss", [(0.0, 1.0), (0.3, 1.0), (1.0, 3.0), (2.0, 1.0)])
def test_split_parameter_schedule(dev, t_bubble, t_ss):
    """Algorithm 1: W_bubble = W[:floor(n t_bubble / t_ss)] goes out at full link rate (direct
    transport, the GPU is idle in a bubble), the rest beside computation (staged transport).  The
    cut is rounded down to a bucket boundary; both parts together are the whole snapshot."""
    wl, sizes, plan, staging = setup(dev)
    try:
        L, nb = wl.L, reft.reft_plan_num_buckets(plan)
        shard = fill_shard(wl, 1, dev)
        want = oracle.pack([oracle.as_bytes(t.cpu()) for t in shard])
        cut = reft.reft_plan_split(plan, t_bubble, t_ss)
        assert cut == min(L, int(L * (t_bubble / t_ss)))
        b = reft.reft_plan_bucket_of(plan, cut)
        if cut == L:
            assert b == nb
        else:
            lo, hi = reft.reft_plan_bucket_range(plan, b)
            assert lo <= cut < hi
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        host = torch.full((L,), CANARY, dtype=torch.uint8, pin_memory=True)
        torch.cuda.synchronize()
        reft.reft_snapshot_pack_range(plan, shard, None, host, 0, b, s1, None)        # bubble
        reft.reft_snapshot_pack_range(plan, shard, staging, host, b, nb, s1, s2)      # compute
        reft.reft_snapshot_wait(plan)
        torch.cuda.synchronize()
        assert np.array_equal(host.numpy(), want)
    finally:
        reft.reft_plan_destroy(plan)


def test_completed_and_ongoing_snapshots(dev):
    """Section 4.4: the ongoing snapshot replaces the completed one only when all of it has landed;
    a snapshot that is interrupted half way leaves the completed copy intact and still 'latest'."""
    wl, sizes, plan, staging = setup(dev)
    try:
        L, nb = wl.L, reft.reft_plan_num_buckets(plan)
        state = [fill_shard(wl, s, dev) for s in range(3)]          # three successive states
        want = [oracle.pack([oracle.as_bytes(t.cpu()) for t in st]) for st in state]
        bufs = [torch.full((L,), CANARY, dtype=torch.uint8, pin_memory=True) for _ in range(2)]
        addr = [b.data_ptr() for b in bufs]
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        ck = reft.reft_ckpt_create(plan, bufs[0], bufs[1])
        try:
            assert reft.reft_ckpt_latest(ck) == (None, 0)
            # generation 1: complete
            dst, gen = reft.reft_ckpt_begin(ck)
            assert gen == 1 and dst in addr
            assert reft.reft_ckpt_latest(ck) == (None, 0)           # nothing complete yet
            reft.reft_snapshot_pack(plan, state[0], staging, dst, s1, s2, host_cap=L)
            reft.reft_ckpt_commit(ck, s2)
            s2.synchronize()
            src1, g = reft.reft_ckpt_latest(ck)
            assert (src1, g) == (dst, 1)
            assert np.array_equal(host_view(src1, L), want[0])
            # generation 2: torn (only the first half of the buckets, never committed)
            dst2, gen2 = reft.reft_ckpt_begin(ck)
            assert gen2 == 2 and dst2 != src1
            reft.reft_snapshot_pack_range(plan, state[1], staging, dst2, 0, nb // 2, s1, s2, host_cap=L)
            reft.reft_snapshot_wait(plan)
            torch.cuda.synchronize()
            assert reft.reft_ckpt_latest(ck) == (src1, 1)           # still the completed copy
            assert np.array_equal(host_view(src1, L), want[0])      # and it is intact
            # a new attempt reuses the torn buffer, not the completed one
            dst3, gen3 = reft.reft_ckpt_begin(ck)
            assert gen3 == 3 and dst3 == dst2
            reft.reft_snapshot_pack(plan, state[2], None, dst3, s1, None, host_cap=L)   # direct
            assert reft.reft_ckpt_latest(ck)[1] in (1, 3)           # 1 until the commit lands
            reft.reft_ckpt_commit(ck, s1)
            s1.synchronize()
            assert reft.reft_ckpt_latest(ck) == (dst3, 3)
            assert np.array_equal(host_view(dst3, L), want[2])
            # the next generation overwrites the older complete copy
            dst4, gen4 = reft.reft_ckpt_begin(ck)
            assert gen4 == 4 and dst4 == src1
            assert reft.reft_ckpt_latest(ck) == (dst3, 3)
            with pytest.raises(reft.ReftError):
                reft.reft_ckpt_commit(ck, s1) or reft.reft_ckpt_commit(ck, s1)   # second: no begin
        finally:
            torch.cuda.synchronize()
            reft.reft_ckpt_destroy(ck)
    finally:
        reft.reft_plan_destroy(plan)


def test_begin_is_refused_while_a_commit_is_in_flight(dev):
    """A second snapshot may not begin before the first one's COMPLETED mark has landed: until then
    neither buffer may be overwritten.  The commit is held back from the host by a long sleep kernel
    queued in front of it; every kernel ends normally."""
    wl, sizes, plan, staging = setup(dev)
    try:
        L = wl.L
        shard = fill_shard(wl, 0, dev)
        want = oracle.pack([oracle.as_bytes(t.cpu()) for t in shard])
        bufs = [torch.full((L,), CANARY, dtype=torch.uint8, pin_memory=True) for _ in range(2)]
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        ck = reft.reft_ckpt_create(plan, bufs[0], bufs[1])
        try:
            dst, gen = reft.reft_ckpt_begin(ck)
            reft.reft_snapshot_pack(plan, shard, staging, dst, s1, s2, host_cap=L)
            with torch.cuda.stream(s2):
                torch.cuda._sleep(100_000_000)           # tens of milliseconds in front of the commit
            reft.reft_ckpt_commit(ck, s2)
            with pytest.raises(reft.ReftError) as e:
                reft.reft_ckpt_begin(ck)
            assert e.value.code == reft.REFT_EBUSY
            assert reft.reft_ckpt_latest(ck) == (None, 0)
            reft.reft_ckpt_wait(ck)
            assert reft.reft_ckpt_latest(ck) == (dst, gen)
            assert np.array_equal(host_view(dst, L), want)
            dst2, gen2 = reft.reft_ckpt_begin(ck)        # accepted now, into the other buffer
            assert gen2 == gen + 1 and dst2 != dst
            # destroying with a commit still queued waits for it instead of freeing its flag
            reft.reft_snapshot_pack(plan, shard, staging, dst2, s1, s2, host_cap=L)
            with torch.cuda.stream(s2):
                torch.cuda._sleep(50_000_000)
            reft.reft_ckpt_commit(ck, s2)
        finally:
            reft.reft_ckpt_destroy(ck)
        torch.cuda.synchronize()
        assert np.array_equal(bufs[0].numpy() if dst2 == bufs[0].data_ptr() else bufs[1].numpy(), want)
    finally:
        reft.reft_plan_destroy(plan)


def test_snapshot_wait_covers_calls_on_different_streams(dev):
    """Two range calls of one snapshot that end on different streams: reft_snapshot_wait returns
    only when both have landed."""
    wl, sizes, plan, staging = setup(dev)
    try:
        L, nb = wl.L, reft.reft_plan_num_buckets(plan)
        shard = fill_shard(wl, 2, dev)
        want = oracle.pack([oracle.as_bytes(t.cpu()) for t in shard])
        host = torch.full((L,), CANARY, dtype=torch.uint8, pin_memory=True)
        s1, s2, s3 = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        with torch.cuda.stream(s2):
            torch.cuda._sleep(100_000_000)               # the first call's copies start late
        reft.reft_snapshot_pack_range(plan, shard, staging, host, 0, nb // 2, s1, s2, host_cap=L)
        reft.reft_snapshot_pack_range(plan, shard, None, host, nb // 2, nb, s3, None, host_cap=L)
        reft.reft_snapshot_wait(plan)
        assert np.array_equal(host.numpy(), want)
        torch.cuda.synchronize()
    finally:
        reft.reft_plan_destroy(plan)


@pytest.mark.parametrize("mode", [1, 2, 0])
def test_replayed_copy_graphs_follow_the_data(dev, mode):
    """The staged transport replays its piece copies as a cached hipGraph when a call repeats the
    same tensors and host buffer.  Every replay must move the tensors' current bytes: the data is
    changed between snapshots, eager work and synchronisations lie between the replays, and each
    snapshot and each restore is compared with the oracle."""
    saved = {n: reft.reft_get_tunable(n) for n in ("graph_copies", "dma_min_bytes")}
    reft.reft_set_tunable("graph_copies", mode)
    reft.reft_set_tunable("dma_min_bytes", 0)          # every piece is a copy of its own
    try:
        wl = make_workload(0)
        sizes = span_nbytes(wl)
        shard = fill_shard(wl, 0, dev)
        plan = reft.reft_plan_create(sizes, wl.bucket_nbytes)
        try:
            slot = reft.reft_plan_staging_slot_bytes(plan)
            staging = torch.empty(2 * slot, dtype=torch.uint8, device=dev)
            host = torch.empty(wl.L, dtype=torch.uint8, pin_memory=True)
            fresh = [torch.zeros_like(t) for t in shard]
            s_a, s_b = torch.cuda.Stream(), torch.cuda.Stream()
            for rep in range(5):
                for t in shard:                          # new contents, same addresses
                    t.view(torch.uint8).add_(rep + 1)
                torch.cuda.synchronize()
                want = oracle.pack_bucketed([oracle.as_bytes(t.cpu()) for t in shard], wl.bucket_nbytes)
                reft.reft_snapshot_pack(plan, shard, staging, host, s_a, s_b)
                reft.reft_snapshot_wait(plan)
                assert np.array_equal(host.numpy(), want), f"snapshot {rep}"
                for t in fresh:
                    t.zero_()
                torch.cuda.synchronize()
                reft.reft_restore(plan, host, staging, fresh, s_b, s_a)
                reft.reft_restore_wait(plan)
                for t, w in zip(fresh, oracle.unpack(want, sizes)):
                    assert np.array_equal(oracle.as_bytes(t.cpu()), w), f"restore {rep}"
        finally:
            reft.reft_plan_destroy(plan)
    finally:
        for n, v in saved.items():
            reft.reft_set_tunable(n, v)
