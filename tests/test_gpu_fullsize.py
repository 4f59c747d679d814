"""GPU parity at the full sizes of configurations 1-4, in the launch configuration bench.py times
(staged snapshot, staged restore, write-burst XOR kernels), plus the direct restore.

At 11-15 GB per shard the oracle cannot recompute everything in seconds, so each case checks
  * sampled windows of every output against the oracle, byte for byte: random windows, windows
    straddling span boundaries and bucket boundaries, and the first and last bytes; the oracle gets
    the window's input bytes from plain ``.cpu()`` slices of the source tensors;
  * properties that hold at any size, evaluated over ALL bytes with plain torch ops (not with the
    library): the XOR of all shards' tensors and the parity is zero span by span, the host snapshot
    equals the tensors' bytes span by span, and restored / reconstructed tensors equal the
    originals.
"""
import gc
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2310_12670_amd as reft
from workload import fill_shard, make_workload, span_nbytes

pytestmark = pytest.mark.gpu

WINDOW = 192 * 1024 + 37          # odd, so windows start and end at unaligned offsets


def say(*a):
    print(time.strftime("[%H:%M:%S]"), *a, flush=True)


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the GPU"
    d = torch.device("cuda:0")
    torch.cuda.set_device(d)
    return d


@pytest.fixture(autouse=True)
def cleanup():
    yield
    gc.collect()
    torch.cuda.empty_cache()


def as_u8(t):
    return t.reshape(-1).view(torch.uint8)


def stream_window(tensors, offs, a, b):
    """Bytes [a, b) of a shard's stream, cut from its tensors with torch slicing (no library)."""
    pieces = []
    i = int(np.searchsorted(offs, a, side="right")) - 1
    while a < b:
        while offs[i + 1] <= a:
            i += 1
        e = min(b, int(offs[i + 1]))
        pieces.append(as_u8(tensors[i])[a - int(offs[i]):e - int(offs[i])].cpu().numpy())
        a = e
    return pieces


def sample_windows(wl, offs, rng, n_random=24, n_span=12, n_bucket=12):
    L = wl.L
    wins = [(0, min(L, WINDOW)), (max(0, L - WINDOW), L)]
    for _ in range(n_random):
        a = int(rng.integers(0, L - WINDOW))
        wins.append((a, a + WINDOW))
    inner = offs[1:-1]
    for o in rng.choice(inner, size=min(n_span, len(inner)), replace=False):
        a = max(0, int(o) - WINDOW // 2)
        wins.append((a, min(L, a + WINDOW)))
    bends = np.cumsum(wl.bucket_nbytes)[:-1]
    for o in rng.choice(bends, size=min(n_bucket, len(bends)), replace=False):
        a = max(0, int(o) - WINDOW // 2)
        wins.append((a, min(L, a + WINDOW)))
    return wins


def check_parity_everywhere(shards, parity, offs):
    """Zero-sum over every byte with torch ops: XOR_s tensor_s[t] ^ parity[span t] == 0."""
    for t in range(len(shards[0])):
        a, b = int(offs[t]), int(offs[t + 1])
        if a == b:
            continue
        acc = parity[a:b].clone()
        for sh in shards:
            acc ^= as_u8(sh[t])
        assert not bool(acc.any()), f"parity is not the XOR of the shards in span {t}"


def check_host_equals_tensors(host, tensors, offs, dev):
    """The pinned snapshot equals the tensors' bytes, span by span, over every byte."""
    for t, x in enumerate(tensors):
        a, b = int(offs[t]), int(offs[t + 1])
        if a == b:
            continue
        assert torch.equal(host[a:b].to(dev, non_blocking=False), as_u8(x)), f"host snapshot, span {t}"


def pinned(nbytes):
    try:
        return torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    except RuntimeError as e:       # visible, never silent
        pytest.fail(f"cannot pin {nbytes / 2**30:.1f} GiB of host memory on this box: {e}")


def run_full(dev, cfg, do_reconstruct, with_gemm=False):
    wl = make_workload(cfg)
    k, L = wl.k, wl.L
    sizes = span_nbytes(wl)
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    rng = np.random.default_rng(wl.seed)
    say(f"config {cfg}: k={k} L={L} spans={len(sizes)} buckets={len(wl.bucket_nbytes)} lost={wl.lost}")
    shards = [fill_shard(wl, s, dev) for s in range(k)]
    own, lost = (wl.lost + 1) % k, wl.lost
    plan = reft.reft_plan_create(sizes, wl.bucket_nbytes)
    pplan = reft.reft_plan_create([L], None, reft.reft_plan_max_bucket_bytes(plan))
    try:
        slot = reft.reft_plan_staging_slot_bytes(plan)
        nslots = max(2, min(16, (1 << 30) // slot))
        staging = torch.empty(nslots * slot, dtype=torch.uint8, device=dev)
        pstaging = torch.empty(nslots * reft.reft_plan_staging_slot_bytes(pplan), dtype=torch.uint8,
                               device=dev)
        host, host_par = pinned(L), pinned(L)
        parity = torch.empty(L, dtype=torch.uint8, device=dev)
        s_snap, s_copy, s_xor, s_load = (torch.cuda.Stream() for _ in range(4))
        torch.cuda.synchronize()

        if with_gemm:                        # the training proxy of configuration 3 runs beside
            n = 8192
            A = torch.randn(n, n, device=dev, dtype=torch.bfloat16)
            B = torch.randn(n, n, device=dev, dtype=torch.bfloat16)
            C = torch.empty(n, n, device=dev, dtype=torch.bfloat16)
            for _ in range(400):
                torch.matmul(A, B, out=C)

        # save phase as bench.py runs it: staged snapshot beside the encode, then the parity
        reft.reft_snapshot_pack(plan, shards[own], staging, host, s_snap, s_copy)
        reft.reft_parity_encode(plan, [t for sh in shards for t in sh], k, parity, s_xor)
        s_snap.wait_stream(s_xor)
        reft.reft_snapshot_pack(pplan, [parity], pstaging, host_par, s_snap, s_copy)
        reft.reft_snapshot_wait(plan)
        reft.reft_snapshot_wait(pplan)
        torch.cuda.synchronize()
        say("save phase done")

        # -- sampled windows against the oracle
        wins = sample_windows(wl, offs, rng)
        host_np, hpar_np = host.numpy(), host_par.numpy()
        par_ref = {}
        for (a, b) in wins:
            win = [oracle.pack(stream_window(shards[s], offs, a, b)) for s in range(k)]
            assert np.array_equal(host_np[a:b], win[own]), f"snapshot window [{a},{b})"
            p = oracle.encode(win)
            par_ref[(a, b)] = (p, win)
            assert np.array_equal(parity[a:b].cpu().numpy(), p), f"parity window [{a},{b})"
            assert np.array_equal(hpar_np[a:b], p), f"parity snapshot window [{a},{b})"
        say(f"{len(wins)} oracle windows ok (snapshot, parity, parity snapshot)")

        # -- every byte, with torch
        check_host_equals_tensors(host, shards[own], offs, dev)
        check_parity_everywhere(shards, parity, offs)
        assert torch.equal(host_par.to(dev), parity)
        say("full-size properties ok (host == tensors, zero-sum, parity snapshot)")

        # -- pack + encode in one pass, as bench.py's stage runs it: same parity, and the packed
        #    stream of the own shard (oracle windows; every byte against the host snapshot)
        par_f = torch.empty(L, dtype=torch.uint8, device=dev)
        packed = torch.empty(L, dtype=torch.uint8, device=dev)
        reft.reft_parity_encode_pack(plan, [t for sh in shards for t in sh], k, own, par_f, packed, s_xor)
        s_xor.synchronize()
        for (a, b), (p, win) in par_ref.items():
            assert np.array_equal(par_f[a:b].cpu().numpy(), p), f"fused parity window [{a},{b})"
            assert np.array_equal(packed[a:b].cpu().numpy(), win[own]), f"fused packed window [{a},{b})"
        assert torch.equal(par_f, parity), "fused parity"
        assert torch.equal(packed, host.to(dev)), "fused packed stream"
        del par_f, packed
        say("pack + encode in one pass ok")

        # -- load phase, once with each transport (bench.py times the staged one): restore of the
        #    own shard and of the parity, oracle windows on the restored tensors, every byte with torch
        lstaging = torch.empty(nslots * slot, dtype=torch.uint8, device=dev)
        for mode, stg, pstg, s_cp in (("staged", lstaging, pstaging, s_copy), ("direct", None, None, None)):
            fresh = [torch.empty_like(t) for t in shards[own]]
            parity2 = torch.empty_like(parity)
            for t in fresh:
                t.view(torch.uint8).fill_(0xA5)
            parity2.fill_(0xA5)
            torch.cuda.synchronize()
            reft.reft_restore(plan, host, stg, fresh, s_cp, s_load)
            reft.reft_restore(pplan, host_par, pstg, [parity2], s_cp, s_load)
            reft.reft_restore_wait(plan)
            reft.reft_restore_wait(pplan)
            torch.cuda.synchronize()
            for (a, b), (p, win) in par_ref.items():
                got = oracle.pack(stream_window(fresh, offs, a, b))
                assert np.array_equal(got, win[own]), f"{mode} restore window [{a},{b})"
                assert np.array_equal(parity2[a:b].cpu().numpy(), p), f"{mode} parity restore window [{a},{b})"
            assert all(torch.equal(a, b) for a, b in zip(fresh, shards[own])), f"{mode} restore"
            assert torch.equal(parity2, parity), f"{mode} restore of the parity"
            say(f"{mode} restore ok ({len(par_ref)} oracle windows, every byte with torch)")
        del lstaging
        del fresh
        if do_reconstruct:
            out = [torch.empty_like(t) for t in shards[lost]]
            rows = [None if s == lost else t for s, sh in enumerate(shards) for t in sh]
            reft.reft_reconstruct_spans(plan, rows, k, lost, parity2, out, s_xor)
            s_xor.synchronize()
            assert all(torch.equal(a, b) for a, b in zip(out, shards[lost])), "reconstruct_spans"
            for (a, b), (p, win) in list(par_ref.items())[:16]:
                want = oracle.reconstruct([win[s] for s in range(k) if s != lost], p)
                got = oracle.pack(stream_window(out, offs, a, b))
                assert np.array_equal(got, want), f"reconstruct window [{a},{b})"
            say("restore and reconstruct ok")
    finally:
        reft.reft_plan_destroy(plan)
        reft.reft_plan_destroy(pplan)


def test_config1_pack_and_parity(dev):
    run_full(dev, 1, do_reconstruct=True)


def test_config2_shuffled_small_buckets(dev):
    run_full(dev, 2, do_reconstruct=True)


def test_config3_beside_gemm_proxy(dev):
    run_full(dev, 3, do_reconstruct=True, with_gemm=True)


def try_pin(nbytes, count):
    """``count`` pinned buffers, or None if the box cannot pin that much (nothing is kept then)."""
    bufs = []
    try:
        for _ in range(count):
            bufs.append(torch.empty(nbytes, dtype=torch.uint8, pin_memory=True))
    except RuntimeError:
        bufs.clear()
        gc.collect()
        torch._C._host_emptyCache() if hasattr(torch._C, "_host_emptyCache") else None
        return None
    return bufs


def test_config4_recovery_from_host(dev):
    """Save all k shards and the parity to pinned host memory, lose shard j, restore the k-1
    survivors from the host, decode the lost shard on the GPU; all k shards' tensors must be
    byte-identical to the originals.  Buckets are random odd lengths (not multiples of 16).

    If the box cannot pin k+1 shards (about 139 GB) the survivors pass through the host two at a
    time instead (snapshot, verify, restore, next): every byte still crosses the link both ways;
    the test prints which mode ran."""
    wl = make_workload(4)
    k, L = wl.k, wl.L
    sizes = span_nbytes(wl)
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    rng = np.random.default_rng(wl.seed)
    lost = wl.lost
    say(f"config 4: k={k} L={L} buckets={len(wl.bucket_nbytes)} lost={lost}")
    shards = [fill_shard(wl, s, dev) for s in range(k)]
    plan = reft.reft_plan_create(sizes, wl.bucket_nbytes)
    pplan = reft.reft_plan_create([L], None, 64 << 20)
    try:
        slot = reft.reft_plan_staging_slot_bytes(plan)
        staging = torch.empty(8 * slot, dtype=torch.uint8, device=dev)
        pstaging = torch.empty(8 * reft.reft_plan_staging_slot_bytes(pplan), dtype=torch.uint8, device=dev)
        bufs = try_pin(L, k + 1)
        all_resident = bufs is not None
        if not all_resident:
            bufs = try_pin(L, 3)
            if bufs is None:
                pytest.skip("cannot pin even 3 shards of host memory on this box")
        host_par, hosts = bufs[0], bufs[1:]
        say(f"pinned {len(bufs) * L / 2**30:.1f} GiB: " +
            ("all k shards host-resident at once" if all_resident else
             f"FALLBACK: only {len(hosts)} of {k} shards host-resident at a time"))
        parity = torch.empty(L, dtype=torch.uint8, device=dev)
        s_snap, s_copy, s_xor, s_load = (torch.cuda.Stream() for _ in range(4))
        torch.cuda.synchronize()

        # parity over the k shards, and its snapshot
        reft.reft_parity_encode(plan, [t for sh in shards for t in sh], k, parity, s_xor)
        s_snap.wait_stream(s_xor)
        reft.reft_snapshot_pack(pplan, [parity], pstaging, host_par, s_snap, s_copy)
        reft.reft_snapshot_wait(pplan)
        torch.cuda.synchronize()
        check_parity_everywhere(shards, parity, offs)
        del parity

        # oracle windows (odd bucket boundaries included): expected snapshot bytes and parity
        wins = sample_windows(wl, offs, rng, n_random=10, n_span=8, n_bucket=14)
        ref_win, ref_lost = {}, {}
        for (a, b) in wins:
            win = [oracle.pack(stream_window(shards[s], offs, a, b)) for s in range(k)]
            p = oracle.encode(win)
            assert np.array_equal(host_par.numpy()[a:b], p), f"parity window [{a},{b})"
            ref_win[(a, b)] = win
            ref_lost[(a, b)] = oracle.reconstruct([win[s] for s in range(k) if s != lost], p)
            assert np.array_equal(ref_lost[(a, b)], win[lost])
        say(f"{len(wins)} oracle windows prepared, parity snapshot ok")

        def save(s, hbuf):
            reft.reft_snapshot_pack(plan, shards[s], staging, hbuf, s_snap, s_copy)

        def check_snapshot(s, hbuf):
            hnp = hbuf.numpy()
            for (a, b), win in ref_win.items():
                assert np.array_equal(hnp[a:b], win[s]), f"snapshot {s} window [{a},{b})"

        residency = "all survivors host-resident" if all_resident else \
            f"fallback, {len(hosts)} of {k} shards host-resident at a time"

        def restore(s, hbuf):
            # survivors alternate between the two transports
            staged = s % 2 == 0
            mode = f"{'staged' if staged else 'direct'} restore of shard {s} ({residency})"
            fresh = [torch.empty_like(t) for t in shards[s]]
            reft.reft_restore(plan, hbuf, staging if staged else None, fresh,
                              s_copy if staged else None, s_load)
            reft.reft_restore_wait(plan)
            torch.cuda.synchronize()
            for (a, b), win in ref_win.items():
                assert np.array_equal(oracle.pack(stream_window(fresh, offs, a, b)), win[s]), \
                    f"{mode}: window [{a},{b})"
            assert all(torch.equal(a, b) for a, b in zip(fresh, shards[s])), mode
            shards[s] = fresh                       # the restored copy is the shard from here on
            gc.collect()
            torch.cuda.empty_cache()

        survivors = [s for s in range(k) if s != lost]
        originals_lost = shards[lost]
        if all_resident:
            for s in range(k):
                save(s, hosts[s])
            reft.reft_snapshot_wait(plan)
            for s in range(k):
                check_snapshot(s, hosts[s])
            say("save phase done, snapshots ok")
            for s in survivors:
                restore(s, hosts[s])
        else:
            for i, s in enumerate(survivors):
                hbuf = hosts[i % len(hosts)]
                save(s, hbuf)
                reft.reft_snapshot_wait(plan)
                check_snapshot(s, hbuf)
                restore(s, hbuf)
            say("survivors saved, checked and restored one after another")

        parity2 = torch.empty(L, dtype=torch.uint8, device=dev)
        reft.reft_restore(pplan, host_par, None, [parity2], None, s_load)
        s_load.synchronize()
        out = [torch.empty_like(t) for t in originals_lost]
        rows = [t for s in range(k) for t in (shards[s] if s != lost else [None] * len(sizes))]
        reft.reft_reconstruct_spans(plan, rows, k, lost, parity2, out, s_xor)
        s_xor.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(out, originals_lost)), \
            f"reconstructed shard ({residency})"
        for (a, b), want in ref_lost.items():
            assert np.array_equal(oracle.pack(stream_window(out, offs, a, b)), want), \
                f"reconstruct window [{a},{b}) ({residency})"
        say(f"recovery ok ({residency}): k-1 shards restored from host, lost shard decoded")
    finally:
        reft.reft_plan_destroy(plan)
        reft.reft_plan_destroy(pplan)
