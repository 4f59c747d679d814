"""GPU parity of the rotated parity placement (section 4.2) against the CPU oracle, bit-exact:
every member's unit, and the decode of every possible lost member from the survivors alone."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_12670_amd as reft
from workload import fill_shard, make_workload, span_nbytes

pytestmark = pytest.mark.gpu
CANARY = 0x3C


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the GPU"
    d = torch.device("cuda:0")
    torch.cuda.set_device(d)
    return d


def check_rotated(dev, shards, sizes, losts=None):
    k, L = len(shards), sum(sizes)
    cpu = [[oracle.as_bytes(t.cpu()) for t in sh] for sh in shards]
    streams = [oracle.pack(c) if L else np.zeros(0, np.uint8) for c in cpu]
    plan = reft.reft_plan_create(sizes)
    try:
        Lseg = reft.reft_segment_bytes(plan, k)
        assert Lseg == oracle.segment_bytes(L, k)
        flat = [t for sh in shards for t in sh]
        units = []
        for i in range(k):
            raw = torch.full((Lseg + 512,), CANARY, dtype=torch.uint8, device=dev)
            unit = raw[256:256 + Lseg]
            rows = [None if (s == i) else t for s, sh in enumerate(shards) for t in sh]
            reft.reft_parity_encode_rotated(plan, rows, k, i, unit if Lseg else raw.data_ptr() + 256)
            torch.cuda.synchronize()
            want = oracle.encode_rotated(streams, i)
            assert np.array_equal(unit.cpu().numpy(), want), f"unit of member {i}"
            r = raw.cpu().numpy()
            assert np.all(r[:256] == CANARY) and np.all(r[256 + Lseg:] == CANARY)
            units.append(unit)
        assert sum(u.numel() for u in units) == k * Lseg          # redundancy volume
        for lost in (range(k) if losts is None else losts):
            out = [torch.full_like(t.reshape(-1).view(torch.uint8), CANARY) for t in shards[lost]]
            rows = [None if s == lost else t for s, sh in enumerate(shards) for t in sh]
            pars = [None if s == lost else (units[s] if Lseg else units[s].data_ptr())
                    for s in range(k)]
            reft.reft_reconstruct_rotated(plan, rows, pars, k, lost, out)
            torch.cuda.synchronize()
            want = oracle.reconstruct_rotated(
                [None if s == lost else streams[s] for s in range(k)],
                [None if s == lost else units[s].cpu().numpy() for s in range(k)], lost, L)
            assert np.array_equal(want, streams[lost])
            got = oracle.pack([o.cpu().numpy() for o in out]) if L else np.zeros(0, np.uint8)
            assert np.array_equal(got, want), f"decode of lost member {lost}"
    finally:
        reft.reft_plan_destroy(plan)


def test_config0_every_member_and_every_loss(dev):
    wl = make_workload(0)
    shards = [fill_shard(wl, s, dev) for s in range(wl.k)]
    check_rotated(dev, shards, span_nbytes(wl))


def test_shrunk_config2_eight_members(dev):
    wl = make_workload(2, shrink=8, layers=2)
    shards = [fill_shard(wl, s, dev) for s in range(wl.k)]
    check_rotated(dev, shards, span_nbytes(wl), losts=[0, wl.lost, wl.k - 1])


@pytest.mark.parametrize("k", [2, 3, 5, 8, 11])
@pytest.mark.parametrize("sizes", [[7], [1, 0, 3], [100, 1, 0, 4099, 33, 16], [65536, 17, 262144 + 5],
                                   [5] * 40])
def test_ragged_sizes_and_segment_cuts(dev, k, sizes):
    """Stream lengths that do not divide by k-1 (zero-extended last segment), segments cutting
    through tensors at odd bytes, tiny tensors, more than eight members (chained passes)."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(k * 1000 + len(sizes))
    shards = [[torch.randint(0, 256, (n,), dtype=torch.uint8, device=dev, generator=gen) for n in sizes]
              for _ in range(k)]
    check_rotated(dev, shards, sizes)
