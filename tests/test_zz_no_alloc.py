"""GPU test of reft_parity_encode_noalloc, the entry point for callers that cannot allocate: its
output must equal reft_parity_encode's (and the CPU oracle's) byte for byte, on calls in a row that
share the library's static scratch, the later ones on smaller inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_12670_amd as reft

pytestmark = pytest.mark.gpu
CANARY = 0x6B


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the GPU"
    d = torch.device("cuda:0")
    torch.cuda.set_device(d)
    return d


def make_shards(dev, k, sizes, seed):
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    return [[torch.randint(0, 256, (n,), dtype=torch.uint8, device=dev, generator=gen) for n in sizes]
            for _ in range(k)]


def sizes_for(total, nspans, seed):
    """nspans sizes (multiples of 16 except a ragged last one) that sum to `total`."""
    rng = np.random.default_rng(seed)
    cuts = np.sort(rng.choice(np.arange(1, total // 16), size=nspans - 1, replace=False)) * 16
    edges = np.concatenate([[0], cuts, [total]])
    return [int(b - a) for a, b in zip(edges[:-1], edges[1:])]


def encode_both_ways(dev, k, sizes, seed, stream):
    """(no-alloc output, reft_parity_encode output, oracle output) for one set of shards."""
    L = sum(sizes)
    shards = make_shards(dev, k, sizes, seed)
    flat = [t for sh in shards for t in sh]
    plan = reft.reft_plan_create(sizes, None, 1 << 20)
    try:
        outs = []
        for fn in (reft.reft_parity_encode_noalloc, reft.reft_parity_encode):
            buf = torch.full((L + 512,), CANARY, dtype=torch.uint8, device=dev)
            torch.cuda.synchronize()
            fn(plan, flat, k, buf[256:256 + L], stream)
            torch.cuda.synchronize()
            raw = buf.cpu().numpy()
            assert np.all(raw[:256] == CANARY) and np.all(raw[256 + L:] == CANARY), fn.__name__
            outs.append(raw[256:256 + L].copy())
        streams = [oracle.pack([oracle.as_bytes(t.cpu()) for t in sh]) for sh in shards]
        outs.append(oracle.encode(streams))
        return outs
    finally:
        reft.reft_plan_destroy(plan)


def test_noalloc_encode_equals_encode_on_calls_in_a_row(dev):
    s = torch.cuda.Stream()
    # first call: eight shards of 24 MiB + 5 bytes in 300 spans (write-burst kernel, counters in the
    # static scratch); then smaller ones that reuse the scratch: five shards of 9 MiB in 40 spans
    # (burst kernel again, fewer pointers, fewer rounds), three shards of 70 KB (ordinary kernel),
    # and twelve shards (two chained passes) of 10 MiB
    cases = [(8, sizes_for((24 << 20) + 5, 300, 1), 11), (5, sizes_for((9 << 20) + 16, 40, 2), 12),
             (3, [70001, 0, 33, 4096], 13), (12, sizes_for((10 << 20) + 48, 64, 3), 14),
             (8, sizes_for((24 << 20) + 5, 300, 1), 15)]
    for k, sizes, seed in cases:
        got, ref, want = encode_both_ways(dev, k, sizes, seed, s)
        assert np.array_equal(got, want), f"no-alloc encode differs from the oracle (k={k}, T={len(sizes)})"
        assert np.array_equal(got, ref), f"no-alloc encode differs from reft_parity_encode (k={k})"


def test_noalloc_encode_back_to_back_on_one_stream(dev):
    """Two calls queued on one stream without a synchronisation between them, the second smaller:
    the second call's pointer uploads and counter clearing are ordered behind the first's kernels."""
    s = torch.cuda.Stream()
    k1, sizes1 = 8, sizes_for(20 << 20, 200, 5)
    k2, sizes2 = 6, sizes_for(9 << 20, 17, 6)
    sh1, sh2 = make_shards(dev, k1, sizes1, 21), make_shards(dev, k2, sizes2, 22)
    p1 = reft.reft_plan_create(sizes1, None, 0)
    p2 = reft.reft_plan_create(sizes2, None, 0)
    try:
        o1 = torch.empty(sum(sizes1), dtype=torch.uint8, device=dev)
        o2 = torch.empty(sum(sizes2), dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()
        reft.reft_parity_encode_noalloc(p1, [t for sh in sh1 for t in sh], k1, o1, s)
        reft.reft_parity_encode_noalloc(p2, [t for sh in sh2 for t in sh], k2, o2, s)
        s.synchronize()
        for out, shards in ((o1, sh1), (o2, sh2)):
            want = oracle.encode([oracle.pack([oracle.as_bytes(t.cpu()) for t in sh]) for sh in shards])
            assert np.array_equal(out.cpu().numpy(), want)
    finally:
        reft.reft_plan_destroy(p1)
        reft.reft_plan_destroy(p2)


def test_noalloc_encode_rejects_what_the_scratch_cannot_hold(dev):
    sizes = [16] * 5000                                   # 8 x 5000 = 40000 pointers > 32768
    shards = make_shards(dev, 1, sizes, 31)
    plan = reft.reft_plan_create(sizes, None, 0)
    try:
        out = torch.empty(sum(sizes), dtype=torch.uint8, device=dev)
        with pytest.raises(reft.ReftError) as e:
            reft.reft_parity_encode_noalloc(plan, shards[0] * 8, 8, out)
        assert e.value.code == reft.REFT_ESIZE and "32768" in e.value.message
        reft.reft_parity_encode_noalloc(plan, shards[0] * 6, 6, out)   # 30000 pointers fit
        torch.cuda.synchronize()
        assert not out.any()                              # six copies of one shard cancel
        with pytest.raises(reft.ReftError) as e:
            reft.reft_parity_encode_noalloc(plan, shards[0] * 2, 0, out)
        assert e.value.code == reft.REFT_EINVAL
    finally:
        reft.reft_plan_destroy(plan)


def test_noalloc_encode_replays_in_a_hip_graph(dev):
    """Captured into a HIP graph once (the call allocates nothing and clears its counters with a
    kernel, not a memset node) and replayed four times, the tensors' contents changed and eager
    work and synchronisations between the replays: every replay gives the oracle's parity of the
    current contents."""
    k, sizes = 8, sizes_for((9 << 20) + 5, 12, 9)
    L = sum(sizes)
    shards = make_shards(dev, k, sizes, 41)
    flat = [t for sh in shards for t in sh]
    plan = reft.reft_plan_create(sizes, None, 0)
    try:
        out = torch.empty(L, dtype=torch.uint8, device=dev)
        s = torch.cuda.Stream()
        torch.cuda.synchronize()                                    # the shards are filled
        reft.reft_parity_encode_noalloc(plan, flat, k, out, s)      # first use outside the capture
        s.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=s):
            reft.reft_parity_encode_noalloc(plan, flat, k, out, torch.cuda.current_stream())
        for rep in range(4):
            for t in flat[rep::5]:
                t.add_(rep + 1)                                      # new contents, same addresses
            out.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            want = oracle.encode([oracle.pack([oracle.as_bytes(t.cpu()) for t in sh]) for sh in shards])
            assert np.array_equal(out.cpu().numpy(), want), f"replay {rep}"
        del graph
    finally:
        reft.reft_plan_destroy(plan)
