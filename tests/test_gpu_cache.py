"""GPU tests of the plan's pointer-table cache: many distinct pointer arrays cycled through one
plan on two streams (tables are retired while kernels of both streams may still read them), and
the same array reused across streams.  Expected bytes come from the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_12670_amd as reft

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the GPU"
    d = torch.device("cuda:0")
    torch.cuda.set_device(d)
    return d


def test_forty_pointer_sets_on_two_streams(dev):
    sizes = [40000, 16, 0, 70001, 4096, 123, 262144, 33000] * 4        # T = 32, about 1.7 MB
    T, L = len(sizes), sum(sizes)
    nsets, k = 42, 3
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    sets = [[torch.randint(0, 256, (n,), dtype=torch.uint8, device=dev, generator=gen) for n in sizes]
            for _ in range(nsets)]
    cpu = [oracle.pack([oracle.as_bytes(t.cpu()) for t in sh]) for sh in sets]
    plan = reft.reft_plan_create(sizes, None, 0)
    try:
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        outs, packs, decs = [], [], []
        torch.cuda.synchronize()
        # 40 parities over sliding triples (each a pointer table the plan has not seen), a pack
        # and a fused decode per step: 3 x 40 tables of 1 - 4 rows against a cache of 32 tables
        for i in range(nsets - k + 1):
            st = streams[i % 2]
            rows = [t for j in range(k) for t in sets[i + j]]
            par = torch.empty(L, dtype=torch.uint8, device=dev)
            reft.reft_parity_encode(plan, rows, k, par, st)
            pk = torch.empty(L, dtype=torch.uint8, device=dev)
            reft.reft_pack_device(plan, sets[i], pk, streams[(i + 1) % 2])
            fresh = [torch.empty_like(t) for t in sets[i]]
            lost_rows = [None] * T + rows[T:]
            reft.reft_reconstruct_spans(plan, lost_rows, k, 0, par, fresh, st)
            outs.append(par)
            packs.append(pk)
            decs.append(fresh)
        torch.cuda.synchronize()
        for i, (par, pk, fresh) in enumerate(zip(outs, packs, decs)):
            want = oracle.encode(cpu[i:i + k])
            assert np.array_equal(par.cpu().numpy(), want), f"parity of sets {i}..{i + k - 1}"
            assert np.array_equal(pk.cpu().numpy(), cpu[i]), f"pack of set {i}"
            got = oracle.pack([oracle.as_bytes(t.cpu()) for t in fresh])
            assert np.array_equal(got, oracle.reconstruct(cpu[i + 1:i + k], want)), f"decode of set {i}"
    finally:
        reft.reft_plan_destroy(plan)


def test_one_table_shared_by_many_streams(dev):
    """The same pointer array on six streams in turn (more than a table tracks), then retired by
    forty new ones while its last readers may still run."""
    sizes = [1 << 20, 17, 65536 + 3]
    L = sum(sizes)
    gen = torch.Generator(device=dev)
    gen.manual_seed(9)
    base = [torch.randint(0, 256, (n,), dtype=torch.uint8, device=dev, generator=gen) for n in sizes]
    want = oracle.pack([oracle.as_bytes(t.cpu()) for t in base])
    plan = reft.reft_plan_create(sizes, None, 0)
    try:
        streams = [torch.cuda.Stream() for _ in range(6)]
        outs = []
        torch.cuda.synchronize()
        for rep in range(3):
            for st in streams:
                o = torch.empty(L, dtype=torch.uint8, device=dev)
                reft.reft_pack_device(plan, base, o, st)
                outs.append(o)
        others = []
        for i in range(40):
            sh = [torch.full((n,), i + 1, dtype=torch.uint8, device=dev) for n in sizes]
            o = torch.empty(L, dtype=torch.uint8, device=dev)
            # the fills run on torch's current stream: the pack's stream waits for them (and for
            # nothing else, so the earlier readers of the retired tables may still run)
            streams[i % 6].wait_stream(torch.cuda.current_stream())
            reft.reft_pack_device(plan, sh, o, streams[i % 6])
            others.append((sh, o, i + 1))
        torch.cuda.synchronize()
        for o in outs:
            assert np.array_equal(o.cpu().numpy(), want)
        for sh, o, v in others:
            assert bool((o == v).all())
    finally:
        reft.reft_plan_destroy(plan)
