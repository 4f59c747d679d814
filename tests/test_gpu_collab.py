"""GPU parity of collaborative redundant protection (section 4.2, last paragraph): every member of
the tiny configuration keeps its own snapshot, duplicates of peers' shards (ARC) and / or its
rotated parity unit (AEC); for every set of one, two or three lost members the library's recovery
plan is executed with the ordinary calls (reft_restore of a surviving duplicate,
reft_reconstruct_rotated) and compared, byte for byte, with what the CPU oracle recovers from the
same holdings.  What the oracle cannot recover, the plan must refuse (REFT_EUNRECOVERABLE)."""
import itertools

import numpy as np
import pytest
import torch

import oracle
import paper_2310_12670_amd as reft
from workload import fill_shard, make_workload, span_nbytes

pytestmark = pytest.mark.gpu
CANARY = 0x96


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the GPU"
    d = torch.device("cuda:0")
    torch.cuda.set_device(d)
    return d


@pytest.fixture(scope="module")
def group(dev):
    """The save phase, once: snapshots, duplicates for offsets 1..k-1 and parity units of all k
    members (each through the library), plus the oracle's view of the same holdings."""
    wl = make_workload(0)
    k, L, sizes = wl.k, wl.L, span_nbytes(wl)
    shards = [fill_shard(wl, s, dev) for s in range(k)]
    streams = [oracle.pack([oracle.as_bytes(t.cpu()) for t in sh]) for sh in shards]
    plan = reft.reft_plan_create(sizes, wl.bucket_nbytes)
    slot = reft.reft_plan_staging_slot_bytes(plan)
    staging = torch.empty(2 * slot, dtype=torch.uint8, device=dev)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    # member i's duplicate under offset d is a snapshot of shard (i + d) mod k taken by member i
    dup_host = {}
    for d in range(1, k):
        for i in range(k):
            h = torch.empty(L, dtype=torch.uint8, pin_memory=True)
            reft.reft_snapshot_pack(plan, shards[(i + d) % k], staging, h, s1, s2)
            reft.reft_snapshot_wait(plan)
            dup_host[(d, i)] = h
    Lseg = reft.reft_segment_bytes(plan, k)
    units = []
    for i in range(k):
        u = torch.empty(Lseg, dtype=torch.uint8, device=dev)
        rows = [None if s == i else t for s, sh in enumerate(shards) for t in sh]
        reft.reft_parity_encode_rotated(plan, rows, k, i, u, s1)
        units.append(u)
    torch.cuda.synchronize()
    units_cpu = [u.cpu().numpy() for u in units]
    for i in range(k):
        assert np.array_equal(units_cpu[i], oracle.encode_rotated(streams, i))
    yield dict(wl=wl, k=k, L=L, sizes=sizes, shards=shards, streams=streams, plan=plan,
               staging=staging, s1=s1, s2=s2, dup_host=dup_host, units=units, units_cpu=units_cpu)
    reft.reft_plan_destroy(plan)


STRATEGIES = [([1], True), ([1, 2], False), ([], True), ([2], False), ([1, 3], True), ([3, 2], False)]


@pytest.mark.parametrize("offs,aec", STRATEGIES, ids=lambda v: str(v))
def test_every_loss_against_the_oracle(dev, group, offs, aec):
    g = group
    k, L, sizes, plan = g["k"], g["L"], g["sizes"], g["plan"]
    recovered_sets = refused_sets = 0
    for nlost in (1, 2, 3):
        for lost in itertools.combinations(range(k), nlost):
            hide = lambda rows: [None if i in lost else a for i, a in enumerate(rows)]
            dups_cpu = [[g["dup_host"][(d, i)].numpy() for i in range(k)] for d in offs]
            want, unknown, seg = oracle.collab_recover(
                hide(g["streams"]), [hide(r) for r in dups_cpu], offs,
                hide(g["units_cpu"]) if aec else None, lost, L)
            steps, ok = reft.reft_recovery_plan(k, offs, aec, lost)
            assert ok == (unknown == 0), (offs, aec, lost)
            assert sorted(s[0] for s in steps) == [x for x in lost if seg[x].all()], (offs, aec, lost)
            recovered_sets += ok
            refused_sets += not ok
            for member, how, source, which in steps:
                fresh = [torch.full_like(t.reshape(-1).view(torch.uint8), CANARY) for t in g["shards"][member]]
                torch.cuda.synchronize()
                if how == reft.REFT_RECOVER_COPY:
                    assert source not in lost
                    reft.reft_restore(plan, g["dup_host"][(offs[which], source)], g["staging"], fresh,
                                      g["s2"], g["s1"])
                    reft.reft_restore_wait(plan)
                else:
                    rows = [None if s in lost else t for s, sh in enumerate(g["shards"]) for t in sh]
                    pars = [None if s in lost else g["units"][s] for s in range(k)]
                    reft.reft_reconstruct_rotated(plan, rows, pars, k, member, fresh, g["s1"])
                    g["s1"].synchronize()
                got = oracle.pack([f.cpu().numpy() for f in fresh])
                assert np.array_equal(got, want[member]), (offs, aec, lost, member, how)
                assert np.array_equal(got, g["streams"][member])
    assert recovered_sets >= k            # every single loss is recovered by any strategy
    if len(offs) + aec <= 2:
        assert refused_sets >= 1          # three losses are beyond two strategies
