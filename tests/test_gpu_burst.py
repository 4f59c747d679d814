"""GPU parity of the write-burst variant of the XOR kernel against the CPU oracle, bit-exact.

reft_parity_encode and reft_reconstruct_spans switch to this variant by themselves for long
streams with four or more rows; here the thresholds are lowered so that small, ragged cases run
through it as well: every number of sources one launch takes, misaligned sources and
destinations, decode into tensors that are (and are not) aligned alike, stage sizes, grids from
one workgroup up, and with the timing of the bursts switched off (the result must not depend on
it)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_12670_amd as reft
from workload import fill_shard, make_workload, span_nbytes

pytestmark = pytest.mark.gpu
CANARY = 0x5A
GUARD = 512
NAMES = ("burst", "burst_min_rows", "burst_min_bytes", "burst_stage_bytes", "burst_wgs_per_cu",
         "burst_max_polls", "burst_nap", "max_wgs", "unroll", "nontemporal", "small_pieces")


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the GPU"
    d = torch.device("cuda:0")
    torch.cuda.set_device(d)
    return d


@pytest.fixture(autouse=True)
def burst_everywhere():
    saved = {n: reft.reft_get_tunable(n) for n in NAMES}
    reft.reft_set_tunable("burst", 1)
    reft.reft_set_tunable("burst_min_rows", 1)
    reft.reft_set_tunable("burst_min_bytes", 0)
    reft.reft_set_tunable("small_pieces", 0xffffffff)
    yield
    for n, v in saved.items():
        reft.reft_set_tunable(n, v)


def spans_in_arena(sizes, phases, dev, gen):
    starts, pos = [], 0
    for n, ph in zip(sizes, phases):
        starts.append(pos + ph)
        pos += ((n + ph + 255) // 256 + 1) * 256
    arena = torch.randint(0, 256, (max(pos, 256),), dtype=torch.uint8, device=dev, generator=gen)
    return arena, [arena[s:s + n] for s, n in zip(starts, sizes)]


def check_encode(dev, shards, sizes, out_phase=0):
    """Parity of the shards by the library against the oracle's byte loop; canaries around it."""
    k, L = len(shards), sum(sizes)
    streams = [oracle.pack([oracle.as_bytes(t.cpu()) for t in sh]) for sh in shards]
    want = oracle.encode(streams)
    raw = torch.full((L + 2 * GUARD + out_phase,), CANARY, dtype=torch.uint8, device=dev)
    par = raw[GUARD + out_phase:GUARD + out_phase + L]
    plan = reft.reft_plan_create(sizes)
    try:
        reft.reft_parity_encode(plan, [t for sh in shards for t in sh], k, par)
        torch.cuda.synchronize()
    finally:
        reft.reft_plan_destroy(plan)
    r = raw.cpu().numpy()
    assert np.array_equal(r[GUARD + out_phase:GUARD + out_phase + L], want)
    assert np.all(r[:GUARD + out_phase] == CANARY), "wrote before the parity buffer"
    assert np.all(r[GUARD + out_phase + L:] == CANARY), "wrote past the parity buffer"
    return par


def check_decode(dev, shards, sizes, parity, lost, out_phases):
    """Single-loss decode straight into fresh tensors (each between canaries, span t starting
    out_phases[t] bytes after a 256-byte boundary) against the oracle's subtraction decoder."""
    k, L = len(shards), sum(sizes)
    streams = [oracle.pack([oracle.as_bytes(t.cpu()) for t in sh]) for sh in shards]
    want = oracle.reconstruct([streams[s] for s in range(k) if s != lost], oracle.encode(streams))
    assert np.array_equal(want, streams[lost])
    starts, pos = [], GUARD
    for n, ph in zip(sizes, out_phases):
        starts.append(pos + ph)
        pos += ((n + ph + 255) // 256 + 1) * 256
    raw = torch.full((pos + GUARD,), CANARY, dtype=torch.uint8, device=dev)
    outs = [raw[a:a + n] for a, n in zip(starts, sizes)]
    rows = [None if s == lost else t for s, sh in enumerate(shards) for t in sh]
    plan = reft.reft_plan_create(sizes)
    try:
        reft.reft_reconstruct_spans(plan, rows, k, lost, parity, outs)
        torch.cuda.synchronize()
    finally:
        reft.reft_plan_destroy(plan)
    r = raw.cpu().numpy()
    mask = np.ones(r.shape, bool)
    got = []
    for a, n in zip(starts, sizes):
        got.append(r[a:a + n])
        mask[a:a + n] = False
    assert np.array_equal(np.concatenate(got) if got else np.zeros(0, np.uint8), want)
    assert np.all(r[mask] == CANARY), "wrote outside the output tensors"


SIZES = [
    [1], [15], [16], [17], [4095], [4096], [32767], [32768], [32769], [65536 + 3],
    [3, 65533, 16, 131072 + 7, 0, 9],
    [4096 * 5 + 2, 0, 33, 70000, 2, 2, 2, 123457],
    [1 << 20, (1 << 20) + 1, 17],
    [700001, 5, 300007, 1 << 19],
]


@pytest.mark.parametrize("sizes", SIZES, ids=lambda s: "-".join(map(str, s))[:40])
@pytest.mark.parametrize("phase_mode", ["aligned", "mixed", "odd"])
def test_edge_sizes_and_misalignment(dev, sizes, phase_mode):
    gen = torch.Generator(device=dev)
    gen.manual_seed(sum(sizes) + len(sizes))
    rng = np.random.default_rng(len(sizes) + sum(sizes))
    shards, keep = [], []
    for s in range(4):
        if phase_mode == "aligned":
            ph = [0] * len(sizes)
        elif phase_mode == "mixed":
            ph = [int(x) for x in rng.choice([0, 4, 8, 12, 16, 2, 6], size=len(sizes))]
        else:
            ph = [int(x) for x in rng.integers(1, 16, size=len(sizes))]
        arena, spans = spans_in_arena(sizes, ph, dev, gen)
        keep.append(arena)
        shards.append(spans)
    par = check_encode(dev, shards, sizes, out_phase=0 if phase_mode == "aligned" else int(rng.integers(1, 16)))
    # decode into tensors aligned alike relative to the stream (the burst kernel's case) ...
    lost = int(rng.integers(0, 4))
    offs = np.concatenate([[0], np.cumsum(sizes)])
    c = 0 if phase_mode == "aligned" else int(rng.integers(1, 16))
    check_decode(dev, shards, sizes, par, lost, [int((c + o) % 16) for o in offs[:-1]])
    # ... and not alike (falls back to the ordinary kernel; same bytes)
    if phase_mode == "odd":
        check_decode(dev, shards, sizes, par, lost, [int(x) for x in rng.integers(0, 16, size=len(sizes))])


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 15, 16, 23, 31])
def test_every_source_count_of_one_launch_and_chained_passes(dev, k):
    wl = make_workload(0)
    shards = [fill_shard(wl, s % wl.k, dev) for s in range(k)]
    par = check_encode(dev, shards, span_nbytes(wl))
    check_decode(dev, shards, span_nbytes(wl), par, k // 2, [0] * len(wl.spans))


@pytest.mark.parametrize("stage,wgs,max_wgs,polls", [
    (4096, 1, 0, 64), (8192, 2, 1, 64), (16384, 3, 7, 64), (32768, 2, 9, 0), (65536, 1, 0, 64),
    (32768, 2, 0, 0), (32768, 8, 300, 3), (4096, 8, 0, 1),
])
def test_stage_sizes_grids_and_untimed_writes(dev, stage, wgs, max_wgs, polls):
    """Stage size, workgroups per compute unit, grids of fewer than eight workgroups (fewer
    arrival groups) and bursts that never or barely wait: same bytes every time."""
    reft.reft_set_tunable("burst_stage_bytes", stage)
    reft.reft_set_tunable("burst_wgs_per_cu", wgs)
    reft.reft_set_tunable("max_wgs", max_wgs)
    reft.reft_set_tunable("burst_max_polls", polls)
    wl = make_workload(0)
    shards = [fill_shard(wl, s, dev) for s in range(wl.k)]
    par = check_encode(dev, shards, span_nbytes(wl), out_phase=stage % 7)
    check_decode(dev, shards, span_nbytes(wl), par, wl.lost, [0] * len(wl.spans))


@pytest.mark.parametrize("unroll,nt", [(1, 1), (2, 0), (4, 1)])
def test_launch_parameters(dev, unroll, nt):
    reft.reft_set_tunable("unroll", unroll)
    reft.reft_set_tunable("nontemporal", nt)
    wl = make_workload(2, shrink=8, layers=2)
    shards = [fill_shard(wl, s, dev) for s in range(wl.k)]
    check_encode(dev, shards, span_nbytes(wl))


def test_many_small_spans_through_the_piece_walk(dev):
    """Hundreds of spans per stage (the plan-level switch that would keep such plans on the
    ordinary kernel is disabled by the fixture)."""
    rng = np.random.default_rng(5)
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    sizes = [int(x) for x in rng.integers(0, 400, size=3000)] + [200000, 7, 65536]
    shards, keep = [], []
    for s in range(5):
        arena, spans = spans_in_arena(sizes, [int(x) for x in rng.integers(0, 16, size=len(sizes))], dev, gen)
        keep.append(arena)
        shards.append(spans)
    par = check_encode(dev, shards, sizes, out_phase=3)
    offs = np.concatenate([[0], np.cumsum(sizes)])
    check_decode(dev, shards, sizes, par, 2, [int((5 + o) % 16) for o in offs[:-1]])


def test_same_result_as_the_ordinary_kernel_and_back_to_back(dev):
    """Default thresholds on a stream long enough to take the burst kernel by itself; several
    launches in a row share the plan's ring of counter blocks."""
    reft.reft_set_tunable("burst_min_rows", 4)
    reft.reft_set_tunable("burst_min_bytes", 8 << 20)
    reft.reft_set_tunable("small_pieces", 8)
    wl = make_workload(2, shrink=4, layers=2)
    sizes = span_nbytes(wl)
    assert wl.L >= (8 << 20) and wl.k >= 4
    shards = [fill_shard(wl, s, dev) for s in range(wl.k)]
    flat = [t for sh in shards for t in sh]
    plan = reft.reft_plan_create(sizes)
    try:
        outs = [torch.empty(wl.L, dtype=torch.uint8, device=dev) for _ in range(12)]
        for o in outs:
            reft.reft_parity_encode(plan, flat, wl.k, o)
        reft.reft_set_tunable("burst", 0)
        ref = torch.empty(wl.L, dtype=torch.uint8, device=dev)
        reft.reft_parity_encode(plan, flat, wl.k, ref)
        torch.cuda.synchronize()
    finally:
        reft.reft_plan_destroy(plan)
    for o in outs:
        assert torch.equal(o, ref)
    check_decode(dev, shards, sizes, ref, wl.lost, [0] * len(sizes))
    streams = [oracle.pack([oracle.as_bytes(t.cpu()) for t in sh]) for sh in shards]
    assert np.array_equal(ref.cpu().numpy(), oracle.encode(streams))


@pytest.mark.parametrize("L", [1, 15, 16, 17, 4096, 32767, 32768, 32769, 100003, (1 << 20) + 5, 3 * (1 << 20)])
@pytest.mark.parametrize("k,phase", [(1, 0), (3, 0), (4, 5), (7, 11), (9, 3), (16, 0), (31, 7)])
def test_decode_from_packed_streams(dev, L, k, phase):
    """reft_reconstruct (contiguous survivors, parity and output) through the burst variant of the
    contiguous XOR kernel: every source count of one pass, odd addresses, ragged last stage."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(L * 31 + k)
    raws = [torch.randint(0, 256, (L + 64,), dtype=torch.uint8, device=dev, generator=gen) for _ in range(k)]
    streams = [r[(phase * (s + 1)) % 16:][:L] for s, r in enumerate(raws)]
    cpu = [s.cpu().numpy() for s in streams]
    par_np = oracle.encode(cpu)
    praw = torch.full((L + 64,), CANARY, dtype=torch.uint8, device=dev)
    par = praw[(phase * 3) % 16:][:L]
    par.copy_(torch.from_numpy(par_np))
    lost = (L + k) % k
    want = oracle.reconstruct([c for s, c in enumerate(cpu) if s != lost], par_np)
    assert np.array_equal(want, cpu[lost])
    raw = torch.full((L + 2 * GUARD + phase,), CANARY, dtype=torch.uint8, device=dev)
    out = raw[GUARD + phase:GUARD + phase + L]
    got_lost = reft.reft_reconstruct([None if s == lost else t for s, t in enumerate(streams)], par, L, out)
    torch.cuda.synchronize()
    assert got_lost == lost
    r = raw.cpu().numpy()
    assert np.array_equal(r[GUARD + phase:GUARD + phase + L], want)
    assert np.all(r[:GUARD + phase] == CANARY) and np.all(r[GUARD + phase + L:] == CANARY)


def test_a_few_dense_tiles_among_large_spans(dev):
    """Default thresholds: clusters of tiny tensors between large ones (fewer than one tile in a
    hundred is dense in small spans, so the burst kernel walks those stages piece by piece)."""
    reft.reft_set_tunable("burst_min_rows", 4)
    reft.reft_set_tunable("burst_min_bytes", 8 << 20)
    reft.reft_set_tunable("small_pieces", 8)
    rng = np.random.default_rng(11)
    gen = torch.Generator(device=dev)
    gen.manual_seed(11)
    sizes = []
    for _ in range(3):
        sizes += [24 << 20] + [int(x) for x in rng.integers(1, 3000, size=20)]
    shards, keep = [], []
    for s in range(4):
        arena, spans = spans_in_arena(sizes, [0] * len(sizes), dev, gen)
        keep.append(arena)
        shards.append(spans)
    par = check_encode(dev, shards, sizes)
    offs = np.concatenate([[0], np.cumsum(sizes)])
    check_decode(dev, shards, sizes, par, 1, [int(o % 16) for o in offs[:-1]])


def test_concurrent_launches_on_several_streams(dev):
    """Burst kernels of three plans queued on three streams at once: their persistent grids cannot
    all be resident together, so the timing of the bursts breaks down - the bytes must not."""
    reft.reft_set_tunable("burst_min_rows", 4)
    reft.reft_set_tunable("burst_min_bytes", 8 << 20)
    reft.reft_set_tunable("small_pieces", 8)
    wl = make_workload(2, shrink=4, layers=2)
    sizes = span_nbytes(wl)
    shards = [fill_shard(wl, s, dev) for s in range(wl.k)]
    flat = [t for sh in shards for t in sh]
    streams = [oracle.pack([oracle.as_bytes(t.cpu()) for t in sh]) for sh in shards]
    want = oracle.encode(streams)
    plans = [reft.reft_plan_create(sizes) for _ in range(3)]
    sts = [torch.cuda.Stream() for _ in range(3)]
    outs = [[torch.empty(wl.L, dtype=torch.uint8, device=dev) for _ in range(4)] for _ in range(3)]
    try:
        torch.cuda.synchronize()
        for rep in range(4):
            for p, s, o in zip(plans, sts, outs):
                reft.reft_parity_encode(p, flat, wl.k, o[rep], s)
        torch.cuda.synchronize()
    finally:
        for p in plans:
            reft.reft_plan_destroy(p)
    for o in outs:
        for t in o:
            assert np.array_equal(t.cpu().numpy(), want)


def test_burst_statistics_add_up(dev):
    """reft_plan_burst_stats: every writer-wave round of the last burst launch is counted once, as
    met, timed out or not waited; with waiting switched off nothing is counted."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(77)
    sizes = [13 << 20, 12345, 1 << 20, 27 << 20]
    L, k = sum(sizes), 6
    shards = [[torch.randint(0, 256, (n,), dtype=torch.uint8, device=dev, generator=gen) for n in sizes]
              for _ in range(k)]
    want = oracle.encode([oracle.pack([oracle.as_bytes(t.cpu()) for t in sh]) for sh in shards])
    plan = reft.reft_plan_create(sizes)
    try:
        assert reft.reft_plan_burst_stats(plan) == (0, 0, 0, 0)          # nothing launched yet
        out = torch.empty(L, dtype=torch.uint8, device=dev)
        stage = reft.reft_get_tunable("burst_stage_bytes")
        nstages = -(-L // stage)
        for polls in (6, 1, 0):
            reft.reft_set_tunable("burst_max_polls", polls)
            out.zero_()
            reft.reft_parity_encode(plan, [t for sh in shards for t in sh], k, out)
            met, late, skipped, groups = reft.reft_plan_burst_stats(plan)
            assert np.array_equal(out.cpu().numpy(), want), polls
            if polls == 0:
                assert (met, late, skipped, groups) == (0, 0, 0, 0)
            else:
                # one writer-wave round per workgroup and round of the persistent grid (workgroup b
                # takes stages b, b + grid, ...): at least one per stage, less than a grid more
                assert nstages <= met + late + skipped < nstages + 2048, (polls, met, late, skipped)
                assert groups >= 1
    finally:
        reft.reft_plan_destroy(plan)


@pytest.mark.parametrize("k", [1, 2, 5, 8, 11])
@pytest.mark.parametrize("phases", ["alike", "apart"])
def test_fused_pack_and_encode(dev, k, phases):
    """reft_parity_encode_pack: parity of k shards and the packed stream of each shard in turn,
    against the oracle; ragged sizes, misaligned sources; destinations aligned alike (single pass
    where k <= 8) and apart (two launches), canaries around both."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(500 + k)
    rng = np.random.default_rng(k)
    sizes = [3 << 20, 12345, 0, 1 << 20, 17, (2 << 20) + 3, 65536]
    L = sum(sizes)
    shards, keep = [], []
    for s in range(k):
        arena, spans = spans_in_arena(sizes, [int(x) for x in rng.integers(0, 16, size=len(sizes))], dev, gen)
        keep.append(arena)
        shards.append(spans)
    streams = [oracle.pack([oracle.as_bytes(t.cpu()) for t in sh]) for sh in shards]
    want = oracle.encode(streams)
    plan = reft.reft_plan_create(sizes)
    try:
        for own in sorted({0, k // 2, k - 1}):
            ph_a = int(rng.integers(0, 16))
            ph_b = ph_a if phases == "alike" else (ph_a + 1 + int(rng.integers(0, 15))) % 16
            ra = torch.full((L + 2 * GUARD + ph_a,), CANARY, dtype=torch.uint8, device=dev)
            rb = torch.full((L + 2 * GUARD + ph_b,), CANARY, dtype=torch.uint8, device=dev)
            par, pk = ra[GUARD + ph_a:GUARD + ph_a + L], rb[GUARD + ph_b:GUARD + ph_b + L]
            reft.reft_parity_encode_pack(plan, [t for sh in shards for t in sh], k, own, par, pk)
            torch.cuda.synchronize()
            a, b = ra.cpu().numpy(), rb.cpu().numpy()
            assert np.array_equal(a[GUARD + ph_a:GUARD + ph_a + L], want), (k, own, "parity")
            assert np.array_equal(b[GUARD + ph_b:GUARD + ph_b + L], streams[own]), (k, own, "packed")
            assert np.all(a[:GUARD + ph_a] == CANARY) and np.all(a[GUARD + ph_a + L:] == CANARY)
            assert np.all(b[:GUARD + ph_b] == CANARY) and np.all(b[GUARD + ph_b + L:] == CANARY)
        with pytest.raises(reft.ReftError) as e:
            reft.reft_parity_encode_pack(plan, [t for sh in shards for t in sh], k, k, par, pk)
        assert e.value.code == reft.REFT_EINVAL
        with pytest.raises(reft.ReftError) as e:
            reft.reft_parity_encode_pack(plan, [t for sh in shards for t in sh], k, 0, par, pk, packed_cap=L - 1)
        assert e.value.code == reft.REFT_ESIZE
    finally:
        reft.reft_plan_destroy(plan)


@pytest.mark.parametrize("stage,wgs", [(4096, 2), (12288, 1), (36864, 2), (40960, 2)])
def test_fused_pack_and_encode_stage_sizes(dev, stage, wgs):
    """Stage sizes up to the largest whose two images fit the LDS, and one beyond (two launches)."""
    reft.reft_set_tunable("burst_stage_bytes", stage)
    reft.reft_set_tunable("burst_wgs_per_cu", wgs)
    gen = torch.Generator(device=dev)
    gen.manual_seed(stage)
    sizes = [(5 << 20) + 48, 4096, 999]
    L, k = sum(sizes), 6
    shards = [[torch.randint(0, 256, (n,), dtype=torch.uint8, device=dev, generator=gen) for n in sizes]
              for _ in range(k)]
    streams = [oracle.pack([oracle.as_bytes(t.cpu()) for t in sh]) for sh in shards]
    plan = reft.reft_plan_create(sizes)
    try:
        par = torch.empty(L, dtype=torch.uint8, device=dev)
        pk = torch.empty(L, dtype=torch.uint8, device=dev)
        for rep in range(3):                      # back to back on one plan
            reft.reft_parity_encode_pack(plan, [t for sh in shards for t in sh], k, 2, par, pk)
        torch.cuda.synchronize()
        assert np.array_equal(par.cpu().numpy(), oracle.encode(streams))
        assert np.array_equal(pk.cpu().numpy(), streams[2])
    finally:
        reft.reft_plan_destroy(plan)
