"""GPU parity: the HIP path through the C ABI against the CPU oracle, byte for byte.

Every case builds seeded inputs on the GPU, hands the oracle plain ``.cpu()`` copies (never
anything the library produced) and compares all outputs element by element: the bucketed snapshot
in pinned host memory, the packed device stream, the XOR parity read through span tables, the
reconstruction of every (or the seed-chosen) lost shard, and the restored tensors.  Device and host
outputs sit between canary bands that must stay untouched.  The bar is bit-exact.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_12670_amd as reft
from workload import fill_shard, make_workload, span_nbytes

pytestmark = pytest.mark.gpu

GUARD = 512
CANARY = 0xC3
DIRECT = False      # set per test: snapshot / restore without a staging ring (kernels touch host)


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the GPU"
    d = torch.device("cuda:0")
    torch.cuda.set_device(d)
    return d


@pytest.fixture(autouse=True, params=["direct", "staged", "staged-gather", "direct-lds",
                                      "staged-gather-lds", "staged-tiny-dma", "staged-2streams",
                                      "staged-tiny-dma-2streams"])
def default_tunables(request):
    """Every case runs with each host transport: direct (kernels touch pinned host memory),
    staged (large pieces by DMA from the tensors, runs of small pieces through gather kernel and
    staging ring), staged-gather (every byte through the gather kernel and the ring) and
    staged-tiny-dma (every piece, however small, its own DMA copy); "-2streams" alternates the piece
    copies between copy_stream and the plan's helper stream (dma_streams = 2); "-lds" forces the
    kernels' LDS-staged small-piece path on for every tile.  Launch parameters are restored
    afterwards."""
    global DIRECT
    names = ("max_wgs", "nontemporal", "unroll", "tile_shift", "link_wgs", "small_pieces",
             "dma_min_bytes", "gather_min_pieces", "dma_streams")
    saved = {n: reft.reft_get_tunable(n) for n in names}
    DIRECT = request.param.startswith("direct")
    if "-gather" in request.param:
        reft.reft_set_tunable("dma_min_bytes", 1 << 62)
        reft.reft_set_tunable("gather_min_pieces", 1)
    if "-tiny-dma" in request.param:
        reft.reft_set_tunable("dma_min_bytes", 0)
    reft.reft_set_tunable("dma_streams", 2 if request.param.endswith("-2streams") else 1)
    if request.param.endswith("-lds"):
        reft.reft_set_tunable("small_pieces", 0)
    yield
    for n, v in saved.items():
        reft.reft_set_tunable(n, v)


# ------------------------------------------------------------------------------------------------
# helpers
# ------------------------------------------------------------------------------------------------
class Guarded:
    """A device (or pinned host) byte buffer of n bytes between two canary bands."""

    def __init__(self, n, device=None, pinned=False, phase=0):
        total = n + 2 * GUARD + phase
        if pinned:
            self.raw = torch.full((total,), CANARY, dtype=torch.uint8, pin_memory=True)
        else:
            self.raw = torch.full((total,), CANARY, dtype=torch.uint8, device=device)
        self.n = n
        self.start = GUARD + phase
        self.view = self.raw[self.start:self.start + n]

    def check(self, what):
        raw = self.raw.cpu().numpy() if self.raw.is_cuda else self.raw.numpy()
        assert np.all(raw[:self.start] == CANARY), f"{what}: wrote before the buffer"
        assert np.all(raw[self.start + self.n:] == CANARY), f"{what}: wrote past the buffer"

    def bytes(self):
        v = self.view.cpu() if self.view.is_cuda else self.view
        return v.numpy().copy()


def arena_spans(sizes, phases, dev, gen):
    """Spans cut out of one byte arena: span t starts at a 256-byte boundary plus phases[t]."""
    starts, pos = [], 0
    for n, ph in zip(sizes, phases):
        starts.append(pos + ph)
        pos += ((n + ph + 255) // 256 + 1) * 256
    arena = torch.randint(0, 256, (max(pos, 256),), dtype=torch.uint8, device=dev, generator=gen)
    assert arena.data_ptr() % 256 == 0
    return arena, [arena[s:s + n] for s, n in zip(starts, sizes)]


def cpu_bytes(tensors):
    return [oracle.as_bytes(t.cpu()) for t in tensors]


def run_case(dev, shards, sizes, buckets=None, uniform=0, lost=None, nslots=2, out_phase=0,
             fresh_phases=None, seed=0):
    """All entry points on one set of k shards (lists of tensors sharing ``sizes``)."""
    k = len(shards)
    L = sum(sizes)
    T = len(sizes)
    cpu = [cpu_bytes(sh) for sh in shards]
    plan = reft.reft_plan_create(sizes, buckets, uniform)
    try:
        assert reft.reft_plan_stream_bytes(plan) == L
        nb = reft.reft_plan_num_buckets(plan)
        blist = [reft.reft_plan_bucket_range(plan, b) for b in range(nb)]
        blens = [hi - lo for lo, hi in blist]
        streams = [oracle.pack_bucketed(c, blens) if L else np.zeros(0, np.uint8) for c in cpu]

        slot = reft.reft_plan_staging_slot_bytes(plan)
        staging = None if DIRECT else torch.empty(max(256, nslots * slot), dtype=torch.uint8,
                                                  device=dev)
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()

        # S1+S2+S3: snapshot of shard 0 into pinned host memory
        host = Guarded(L, pinned=True)
        reft.reft_snapshot_pack(plan, shards[0], staging, host.view, s1, s2, host_cap=L)
        reft.reft_snapshot_wait(plan)
        assert reft.reft_snapshot_query(plan)
        assert np.array_equal(host.bytes(), streams[0]), "snapshot_pack"
        host.check("snapshot_pack")

        # S1 alone, every shard
        packed = []
        for s in range(k):
            g = Guarded(L, dev, phase=(out_phase * (s + 1)) % 16)
            reft.reft_pack_device(plan, shards[s], g.view, None, dst_cap=L)
            packed.append(g)
        torch.cuda.synchronize()
        for s in range(k):
            assert np.array_equal(packed[s].bytes(), streams[s]), f"pack_device shard {s}"
            packed[s].check("pack_device")

        # S4: parity through the span tables
        parity_ref = oracle.encode(streams)
        par = Guarded(L, dev, phase=out_phase)
        flat = [t for sh in shards for t in sh]
        reft.reft_parity_encode(plan, flat, k, par.view, s1)
        s1.synchronize()
        assert np.array_equal(par.bytes(), parity_ref), "parity_encode"
        par.check("parity_encode")

        # S1+S4 fused: the parity again, and the packed stream of one shard, in one call
        own = k - 1 if lost is None else lost
        par2 = Guarded(L, dev, phase=out_phase)
        pk2 = Guarded(L, dev, phase=out_phase if seed % 2 == 0 else (out_phase + 5) % 16)
        reft.reft_parity_encode_pack(plan, flat, k, own, par2.view, pk2.view, s1, packed_cap=L)
        s1.synchronize()
        assert np.array_equal(par2.bytes(), parity_ref), "parity_encode_pack: parity"
        assert np.array_equal(pk2.bytes(), streams[own]), "parity_encode_pack: packed stream"
        par2.check("parity_encode_pack (parity)")
        pk2.check("parity_encode_pack (packed)")

        # S6: decode the lost shard(s) from the packed survivors and the parity
        for j in (range(k) if lost is None else [lost]):
            out = Guarded(L, dev, phase=out_phase)
            arg = [None if s == j else packed[s].view for s in range(k)]
            got_j = reft.reft_reconstruct(arg, par.view, L, out.view, s2)
            s2.synchronize()
            assert got_j == j
            want = oracle.reconstruct([streams[s] for s in range(k) if s != j], parity_ref)
            assert np.array_equal(out.bytes(), want), f"reconstruct lost={j}"
            assert np.array_equal(want, streams[j])
            out.check("reconstruct")

        gen = torch.Generator(device=dev)
        gen.manual_seed(1000 + seed)
        phases = fresh_phases if fresh_phases is not None else [0] * T

        # S6+S7 fused: decode the lost shard straight into fresh tensors, survivors read in place
        for j in ([k - 1] if lost is None else [lost]):
            arena0, fresh0 = arena_spans(sizes, phases, dev, gen)
            rows = [None if s == j else t for s, sh in enumerate(shards) for t in sh]
            reft.reft_reconstruct_spans(plan, rows, k, j, par.view, fresh0, s1)
            s1.synchronize()
            want = oracle.reconstruct([streams[s] for s in range(k) if s != j], parity_ref)
            for t, (f, w) in enumerate(zip(fresh0, oracle.unpack(want, sizes))):
                assert np.array_equal(f.cpu().numpy(), w), f"reconstruct_spans lost={j} span {t}"

        # S5+S7: restore shard 0 from the host snapshot into fresh tensors
        arena, fresh = arena_spans(sizes, phases, dev, gen)
        before = arena.cpu().numpy().copy()
        reft.reft_restore(plan, host.view, staging, fresh, s2, s1, host_bytes=L)
        reft.reft_restore_wait(plan)
        want_spans = oracle.unpack(streams[0], sizes)
        for t, (f, w) in enumerate(zip(fresh, want_spans)):
            assert np.array_equal(f.cpu().numpy(), w), f"restore span {t}"
        # nothing outside the spans was written
        after = arena.cpu().numpy()
        mask = np.ones(after.size, dtype=bool)
        base = arena.data_ptr()
        for f in fresh:
            o = f.data_ptr() - base
            mask[o:o + f.numel()] = False
        assert np.array_equal(after[mask], before[mask]), "restore wrote outside the spans"

        # S7 alone: scatter the reconstructed / packed stream of shard k-1 into fresh tensors
        arena2, fresh2 = arena_spans(sizes, phases, dev, gen)
        reft.reft_unpack_device(plan, packed[k - 1].view, fresh2, None, src_bytes=L)
        torch.cuda.synchronize()
        want_spans = oracle.unpack(streams[k - 1], sizes)
        for t, (f, w) in enumerate(zip(fresh2, want_spans)):
            assert np.array_equal(f.cpu().numpy(), w), f"unpack_device span {t}"
    finally:
        reft.reft_plan_destroy(plan)


def random_buckets(L, rng, lo, hi):
    out, left = [], L
    while left:
        n = min(left, 2 * int(rng.integers(lo, hi)) + 1)
        out.append(n)
        left -= n
    return out


# ------------------------------------------------------------------------------------------------
# the configurations
# ------------------------------------------------------------------------------------------------
def test_config0_every_lost_shard(dev):
    wl = make_workload(0)
    shards = [fill_shard(wl, s, dev) for s in range(wl.k)]
    run_case(dev, shards, span_nbytes(wl), wl.bucket_nbytes, lost=None)


@pytest.mark.parametrize("cfg,shrink,layers", [(1, 8, 2), (2, 8, 3), (3, 8, 2), (4, 8, 2)])
def test_shrunk_configs(dev, cfg, shrink, layers):
    """Each Llama-shaped configuration at a size the oracle finishes in seconds: several tiles per
    span, ragged tails, the configuration's own span order and bucket rule."""
    wl = make_workload(cfg, shrink=shrink, layers=layers)
    shards = [fill_shard(wl, s, dev) for s in range(wl.k)]
    run_case(dev, shards, span_nbytes(wl), wl.bucket_nbytes, lost=wl.lost, seed=cfg)


@pytest.mark.parametrize("buckets", ["one", "tiny_odd", "uniform_4k", "uniform_1m"])
def test_bucket_independence_on_config0(dev, buckets):
    wl = make_workload(0)
    rng = np.random.default_rng(3)
    shards = [fill_shard(wl, s, dev) for s in range(2)]
    if buckets == "one":
        run_case(dev, shards, span_nbytes(wl), None, 0, lost=1)
    elif buckets == "tiny_odd":
        run_case(dev, shards, span_nbytes(wl), random_buckets(wl.L, rng, 20000, 90000), lost=0,
                 nslots=3)
    elif buckets == "uniform_4k":
        sub = fill_shard(make_workload(0, shrink=8), 0, dev)
        sizes = [t.numel() * t.element_size() for t in sub]
        run_case(dev, [sub, fill_shard(make_workload(0, shrink=8), 1, dev)], sizes, None, 4096,
                 lost=1, nslots=4)
    else:
        run_case(dev, shards, span_nbytes(wl), None, 1 << 20, lost=0, nslots=1)


# ------------------------------------------------------------------------------------------------
# alignment, raggedness and degenerate sizes
# ------------------------------------------------------------------------------------------------
EDGE_SIZES = [
    [1],
    [15], [16], [17],
    [0, 0, 5, 0],
    [1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1],
    [65535], [65536], [65537],
    [65536, 65536],
    [3, 65533, 16, 131072 + 7, 0, 9],
    [4096 * 5 + 2, 0, 33, 70000, 2, 2, 2, 123457],
    [1 << 20, (1 << 20) + 1, 17],
]


@pytest.mark.parametrize("sizes", EDGE_SIZES, ids=lambda s: "-".join(map(str, s))[:40])
@pytest.mark.parametrize("phase_mode", ["aligned", "mixed", "odd"])
def test_edge_sizes_and_misalignment(dev, sizes, phase_mode):
    gen = torch.Generator(device=dev)
    gen.manual_seed(sum(sizes) + len(sizes))
    rng = np.random.default_rng(len(sizes))
    k = 3
    shards, keep = [], []
    for s in range(k):
        if phase_mode == "aligned":
            ph = [0] * len(sizes)
        elif phase_mode == "mixed":
            ph = [int(x) for x in rng.choice([0, 4, 8, 12, 16, 2, 6], size=len(sizes))]
        else:
            ph = [int(x) for x in rng.integers(1, 16, size=len(sizes))]
        arena, spans = arena_spans(sizes, ph, dev, gen)
        keep.append(arena)
        shards.append(spans)
    L = sum(sizes)
    buckets = random_buckets(L, rng, 1, 40000) if L > 1 else None
    fresh_ph = None if phase_mode == "aligned" else [int(x) for x in rng.integers(0, 16, size=len(sizes))]
    out_phase = 0 if phase_mode == "aligned" else int(rng.integers(1, 16))
    run_case(dev, shards, sizes, buckets, lost=None, nslots=2, out_phase=out_phase,
             fresh_phases=fresh_ph)


@pytest.mark.parametrize("mean_size,tile_shift", [(100, 18), (700, 16), (3000, 18), (40, 14)])
def test_thousands_of_tiny_spans(dev, mean_size, tile_shift):
    """Many small tensors end to end: hundreds to thousands of spans per tile (several LDS passes
    per tile), zero-length spans, odd sizes and odd addresses, next to a few large spans."""
    reft.reft_set_tunable("tile_shift", tile_shift)
    rng = np.random.default_rng(mean_size)
    gen = torch.Generator(device=dev)
    gen.manual_seed(mean_size)
    T = 6000
    sizes = [int(x) for x in rng.integers(0, 2 * mean_size, size=T)]
    for i in rng.choice(T, size=T // 10, replace=False):
        sizes[i] = 0
    for i in rng.choice(T, size=5, replace=False):
        sizes[i] = int(rng.integers(200000, 600000))
    k = 3
    shards, keep = [], []
    for s in range(k):
        ph = [int(x) for x in rng.integers(0, 16, size=T)] if s else [0] * T
        arena, spans = arena_spans(sizes, ph, dev, gen)
        keep.append(arena)
        shards.append(spans)
    L = sum(sizes)
    run_case(dev, shards, sizes, random_buckets(L, rng, 30000, 400000), lost=1, nslots=2,
             out_phase=int(rng.integers(0, 16)),
             fresh_phases=[int(x) for x in rng.integers(0, 16, size=T)])


def test_empty_stream(dev):
    """All spans empty: L = 0, every call succeeds and moves nothing."""
    plan = reft.reft_plan_create([0, 0, 0])
    try:
        assert reft.reft_plan_stream_bytes(plan) == 0 and reft.reft_plan_num_buckets(plan) == 0
        host = Guarded(0, pinned=True)
        out = Guarded(0, dev)
        reft.reft_snapshot_pack(plan, [None] * 3, None, host.view, staging_bytes=0, host_cap=0)
        reft.reft_snapshot_wait(plan)
        reft.reft_parity_encode(plan, [None] * 6, 2, out.view)
        reft.reft_pack_device(plan, [None] * 3, out.view, dst_cap=0)
        reft.reft_unpack_device(plan, out.view, [None] * 3, src_bytes=0)
        reft.reft_restore(plan, host.view, None, [None] * 3, host_bytes=0, staging_bytes=0)
        reft.reft_restore_wait(plan)
        # (an empty torch view reports a null data_ptr, so the survivor's address is given as int)
        assert reft.reft_reconstruct([None, out.raw.data_ptr()], out.raw.data_ptr(), 0,
                                     out.raw.data_ptr()) == 0
        torch.cuda.synchronize()
        host.check("empty")
        out.check("empty")
    finally:
        reft.reft_plan_destroy(plan)


@pytest.mark.parametrize("k", [1, 2, 5, 8, 9, 15, 16, 17, 31, 32])
def test_shard_counts_including_chained_passes(dev, k):
    """k beyond eight sources is folded in several passes; the result is the same XOR."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(k)
    sizes = [70001, 0, 4099, 262144 + 16]
    L = sum(sizes)
    shards, keep = [], []
    for s in range(k):
        arena, spans = arena_spans(sizes, [0, 0, (s % 3) * 4, 0], dev, gen)
        keep.append(arena)
        shards.append(spans)
    cpu = [cpu_bytes(sh) for sh in shards]
    streams = [oracle.pack(c) for c in cpu]
    parity_ref = oracle.encode(streams)
    plan = reft.reft_plan_create(sizes)
    try:
        par = Guarded(L, dev)
        reft.reft_parity_encode(plan, [t for sh in shards for t in sh], k, par.view)
        torch.cuda.synchronize()
        assert np.array_equal(par.bytes(), parity_ref)
        par.check("parity_encode")
        if k <= 31:
            j = k // 3
            arena0, fresh0 = arena_spans(sizes, [4, 0, 0, 9], dev, gen)
            rows = [None if s == j else t for s, sh in enumerate(shards) for t in sh]
            reft.reft_reconstruct_spans(plan, rows, k, j, par.view, fresh0)
            torch.cuda.synchronize()
            for f, w in zip(fresh0, cpu[j]):
                assert np.array_equal(f.cpu().numpy(), w), ("reconstruct_spans", k)
            packed = []
            for s in range(k):
                buf = torch.empty(L, dtype=torch.uint8, device=dev)
                reft.reft_pack_device(plan, shards[s], buf)
                packed.append(buf)
            for j in sorted({0, k // 2, k - 1}):
                out = Guarded(L, dev)
                reft.reft_reconstruct([None if s == j else packed[s] for s in range(k)], par.view,
                                      L, out.view)
                torch.cuda.synchronize()
                want = oracle.reconstruct([streams[s] for s in range(k) if s != j], parity_ref)
                assert np.array_equal(out.bytes(), want), (k, j)
                out.check("reconstruct")
    finally:
        reft.reft_plan_destroy(plan)


def test_float_bit_patterns_survive(dev):
    """NaN payloads, infinities, signed zeros and denormals are moved and XORed as bits."""
    pats = torch.tensor([0x7FC00123, -0x3F0012, 0x7F800000, -0x800000, -0x80000000, 1,
                         0x7F800001, 0x00400000] * 300, dtype=torch.int32, device=dev)
    halves = torch.tensor([0x7FC1, -0x80, -0x8000, 1] * 301, dtype=torch.int16, device=dev)
    k = 4
    shards = []
    for s in range(k):
        a = torch.roll(pats, s).view(torch.float32).clone()
        b = torch.roll(halves, 2 * s + 1).view(torch.bfloat16).clone()
        shards.append([b, a, b.clone(), a.clone()])
    sizes = [t.numel() * t.element_size() for t in shards[0]]
    run_case(dev, shards, sizes, None, 5000, lost=None)


# ------------------------------------------------------------------------------------------------
# launch parameters
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("unroll", [1, 2, 4])
@pytest.mark.parametrize("nt", [0, 1])
@pytest.mark.parametrize("max_wgs,tile_shift", [(0, 16), (1, 12), (7, 14), (64, 20)])
def test_launch_parameters_do_not_change_results(dev, unroll, nt, max_wgs, tile_shift):
    reft.reft_set_tunable("link_wgs", 3 if max_wgs == 7 else 32)
    reft.reft_set_tunable("unroll", unroll)
    reft.reft_set_tunable("nontemporal", nt)
    reft.reft_set_tunable("max_wgs", max_wgs)
    reft.reft_set_tunable("tile_shift", tile_shift)
    wl = make_workload(0, shrink=2)
    shards = [fill_shard(wl, s, dev) for s in range(3)]
    run_case(dev, shards, span_nbytes(wl), None, 300001, lost=1, nslots=2)


# ------------------------------------------------------------------------------------------------
# error behaviour on the GPU machine
# ------------------------------------------------------------------------------------------------
def test_size_and_argument_errors(dev):
    sizes = [1000, 24]
    plan = reft.reft_plan_create(sizes, None, 512)
    try:
        spans = [torch.zeros(n, dtype=torch.uint8, device=dev) for n in sizes]
        staging = torch.empty(4096, dtype=torch.uint8, device=dev)
        host = torch.empty(2048, dtype=torch.uint8, pin_memory=True)
        out = torch.empty(1024, dtype=torch.uint8, device=dev)
        with pytest.raises(reft.ReftError) as e:      # host buffer too small
            reft.reft_snapshot_pack(plan, spans, staging, host, host_cap=1023)
        assert e.value.code == reft.REFT_ESIZE
        with pytest.raises(reft.ReftError) as e:      # staging smaller than one slot
            reft.reft_snapshot_pack(plan, spans, staging, host, staging_bytes=512)
        assert e.value.code == reft.REFT_ESIZE
        with pytest.raises(reft.ReftError) as e:      # direct path needs pinned host memory
            reft.reft_snapshot_pack(plan, spans, None, np.zeros(2048, np.uint8))
        assert e.value.code == reft.REFT_EINVAL
        with pytest.raises(reft.ReftError) as e:      # restore of a snapshot of another length
            reft.reft_restore(plan, host, staging, spans, host_bytes=1025)
        assert e.value.code == reft.REFT_ESIZE
        with pytest.raises(reft.ReftError) as e:      # a non-empty span without a pointer
            reft.reft_pack_device(plan, [spans[0], None], out)
        assert e.value.code == reft.REFT_EINVAL
        with pytest.raises(reft.ReftError) as e:
            reft.reft_pack_device(plan, spans, out, dst_cap=100)
        assert e.value.code == reft.REFT_ESIZE
        with pytest.raises(reft.ReftError) as e:
            reft.reft_parity_encode(plan, spans * 40, 40, out)
        assert e.value.code == reft.REFT_EINVAL
        with pytest.raises(reft.ReftError) as e:      # two shards lost
            reft.reft_reconstruct([None, out, None], out, 1024, out)
        assert e.value.code == reft.REFT_EUNRECOVERABLE
        # the plan still works after the refused calls
        reft.reft_pack_device(plan, spans, out)
        torch.cuda.synchronize()
        assert not out.cpu().numpy().any()
    finally:
        reft.reft_plan_destroy(plan)


def test_back_to_back_snapshots_reuse_the_staging_ring(dev):
    """Several snapshots and restores in flight on the same plan and ring: slot events must order
    every reuse (no synchronisation between the calls)."""
    wl = make_workload(0, shrink=2)
    sizes = span_nbytes(wl)
    L = wl.L
    shards = [fill_shard(wl, s, dev) for s in range(3)]
    plan = reft.reft_plan_create(sizes, None, 100003)
    try:
        slot = reft.reft_plan_staging_slot_bytes(plan)
        staging = None if DIRECT else torch.empty(2 * slot, dtype=torch.uint8, device=dev)
        hosts = [Guarded(L, pinned=True) for _ in range(6)]
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        for i, h in enumerate(hosts):
            reft.reft_snapshot_pack(plan, shards[i % 3], staging, h.view, s1, s2, host_cap=L)
        reft.reft_snapshot_wait(plan)
        torch.cuda.synchronize()
        for i, h in enumerate(hosts):
            want = oracle.pack(cpu_bytes(shards[i % 3]))
            assert np.array_equal(h.bytes(), want), i
            h.check("snapshot")
    finally:
        reft.reft_plan_destroy(plan)
