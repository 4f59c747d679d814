#!/usr/bin/env python3
"""Benchmark of the in-memory checkpointing hot path on one MI355X.

One *step* is one pass of the whole path over one rank-shaped synthetic state, inputs resident in
HBM before the clock starts:

  save   reft_snapshot_pack   own shard   -> pinned host   (staged transport: DMA copies straight
                                                            from the tensors, gather kernel only
                                                            for runs of small tensors)
         reft_parity_encode   k shards    -> parity (device)                  (k-way XOR, in place)
         reft_snapshot_pack   parity      -> pinned host
  load   reft_restore         host shard  -> fresh tensors  (staged transport as well; it starts as
                                                             soon as the shard's snapshot has
                                                             landed and shares the link with the
                                                             parity's snapshot, full duplex)
         reft_restore         host parity -> device
         reft_reconstruct_spans  k-1 survivors + parity -> lost shard's tensors (k-way XOR)

``value`` is the step's checkpoint traffic, 4*L bytes (shard + parity saved to host, shard + parity
loaded back), divided by the step time: the path is bound by the host link, which is why the
HBM-bound kernels are reported separately under ``stages`` and ``roofline``.

The last line printed is the JSON record.  ``python bench.py --help`` lists the options.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0           # MI355X HBM3E, published
LINK_PEAK_GBPS = 63.0            # PCIe Gen5 x16, one direction: 32 GT/s * 16 * 128/130 / 8


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawTextHelpFormatter)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=1, help="workload configuration 0..4 (default 1)")
    ap.add_argument("--gemm-seconds", type=float, default=0.0,
                    help="length of the bf16 GEMM proxy loop for the slowdown figure "
                         "(0 = as long as one save phase; negative = skip)")
    ap.add_argument("--snapshot-wgs", type=int, default=0,
                    help="cap on workgroups of the snapshot kernels while the GEMM proxy runs")
    ap.add_argument("--save-path", choices=["direct", "staged"], default="staged",
                    help="snapshot transport. staged: staging ring + hipMemcpyAsync on the DMA "
                         "engines (what runs beside training); direct: the gather kernel stores "
                         "to pinned host memory itself")
    ap.add_argument("--load-path", choices=["direct", "staged"], default="staged",
                    help="restore transport. staged (default): runtime copies, which share the link "
                         "well with the parity snapshot going the other way; direct: the scatter "
                         "kernel reads pinned host memory itself (fastest when nothing else runs)")
    ap.add_argument("--no-overlap-load", action="store_true",
                    help="start the load phase only when the whole save phase has landed (default: "
                         "the own shard's restore starts as soon as its snapshot is on the host, "
                         "beside the parity's snapshot, which uses the link's other direction)")
    ap.add_argument("--dma-streams", type=int, default=0, choices=[0, 1, 2],
                    help="staged transport: 2 = piece copies alternate with a helper stream "
                         "(0 = library default)")
    ap.add_argument("--one-stream-save", action="store_true",
                    help="staged save: gather kernels and copies in order on one stream")
    ap.add_argument("--two-stream-load", action="store_true",
                    help="staged load: copies and scatter kernels on two streams (default: in order "
                         "on one, which keeps the process within its four hardware queues)")
    ap.add_argument("--staging-mib", type=int, default=1024,
                    help="size of each staging ring in MiB (split into bucket-sized slots)")
    ap.add_argument("--link-wgs", type=int, default=0,
                    help="cap on workgroups of the link-bound kernels (0 = library default)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain device-to-device copy of 1 GiB (torch), the kernel of "
                         "known size that scales the rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    ap.add_argument("--overlap-encode", action="store_true",
                    help="start the own shard's snapshot first and run the parity encode beside it")
    ap.add_argument("--graph-copies", type=int, default=-1, choices=[-1, 0, 1, 2],
                    help="tunable graph_copies: staged piece copies as a replayed hipGraph "
                         "(0 off, 1 independent nodes, 2 chain)")
    ap.add_argument("--no-burst", action="store_true",
                    help="XOR kernels without write bursts (the ordinary gather kernel), for comparison")
    ap.add_argument("--burst-polls", type=int, default=-1,
                    help="tunable burst_max_polls (0 = write bursts are not timed)")
    ap.add_argument("--burst-nap", type=int, default=-1, help="tunable burst_nap")
    ap.add_argument("--burst-stage", type=int, default=0, help="tunable burst_stage_bytes")
    ap.add_argument("--burst-wgs", type=int, default=0, help="tunable burst_wgs_per_cu")
    ap.add_argument("--no-stages", action="store_true", help="skip the per-stage measurements")
    ap.add_argument("--has-demo", action="store_true",
                    help="instead of the benchmark: run a synthetic pipeline-stage timeline (idle "
                         "bubble, then a GEMM burst) with no snapshot, with the whole save phase "
                         "beside compute, and with the bubble-aware split of Algorithm 1; prints "
                         "one JSON line of iteration times")
    ap.add_argument("--no-has", action="store_true",
                    help="skip the short stage-timeline run whose result goes into the record")
    ap.add_argument("--bubble-ms", type=float, default=100.0, help="--has-demo: bubble length")
    ap.add_argument("--burst-gemms", type=int, default=800, help="--has-demo: GEMMs per iteration")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-mib", type=int, default=2048,
                    help="bytes per shard of the CPU-oracle sample, MiB")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU (the simulated node's k shards live in one "
              "GPU's HBM); --gpus N with N > 1 is not supported.", file=sys.stderr)
        return 2

    import torch

    import paper_2310_12670_amd as reft
    from workload import fill_shard, make_workload, span_nbytes

    assert torch.cuda.is_available(), "bench.py needs the GPU (there is no CPU path)"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = make_workload(args.config)
    k, L, T = wl.k, wl.L, len(wl.spans)
    sizes = span_nbytes(wl)
    lost = wl.lost
    own = (lost + 1) % k
    log(f"[bench] config {wl.cfg}: {wl.description}; k={k} T={T} L={L} buckets={len(wl.bucket_nbytes)} "
        f"lost={lost} own={own}")

    t0 = time.time()
    shards = [fill_shard(wl, s, dev) for s in range(k)]
    torch.cuda.synchronize()
    log(f"[bench] generated {k * L / 1e9:.1f} GB of state in {time.time() - t0:.1f} s")

    plan = reft.reft_plan_create(sizes, wl.bucket_nbytes)
    bucket = reft.reft_plan_max_bucket_bytes(plan)
    pplan = reft.reft_plan_create([L], None, bucket)           # the parity as a 1-span shard
    save_staged = args.save_path == "staged"
    load_staged = args.load_path == "staged"
    def ring(p, use):
        if not use:
            return None
        slot = reft.reft_plan_staging_slot_bytes(p)
        nslots = max(2, min(64, (args.staging_mib << 20) // slot))
        return torch.empty(nslots * slot, dtype=torch.uint8, device=dev)
    stag_save, stag_psave = ring(plan, save_staged), ring(pplan, save_staged)
    stag_load, stag_pload = ring(plan, load_staged), ring(pplan, load_staged)
    t0 = time.time()
    host_snap = torch.empty(L, dtype=torch.uint8, pin_memory=True)
    host_par = torch.empty(L, dtype=torch.uint8, pin_memory=True)
    log(f"[bench] pinned {2 * L / 1e9:.1f} GB of host memory in {time.time() - t0:.1f} s")
    parity = torch.empty(L, dtype=torch.uint8, device=dev)
    parity2 = torch.empty(L, dtype=torch.uint8, device=dev)
    fresh_own = [torch.empty_like(t) for t in shards[own]]
    fresh_lost = [torch.empty_like(t) for t in shards[lost]]

    p_own = reft.ptr_array(shards[own])
    p_all = reft.ptr_array([t for sh in shards for t in sh])
    p_surv = reft.ptr_array([None if s == lost else t for s, sh in enumerate(shards) for t in sh])
    p_fresh_own = reft.ptr_array(fresh_own)
    p_fresh_lost = reft.ptr_array(fresh_lost)
    p_par = reft.ptr_array([parity])
    p_par2 = reft.ptr_array([parity2])

    if args.link_wgs:
        reft.reft_set_tunable("link_wgs", args.link_wgs)
    if args.dma_streams:
        reft.reft_set_tunable("dma_streams", args.dma_streams)
    if args.no_burst:
        reft.reft_set_tunable("burst", 0)
    if args.graph_copies >= 0:
        reft.reft_set_tunable("graph_copies", args.graph_copies)
    if args.burst_polls >= 0:
        reft.reft_set_tunable("burst_max_polls", args.burst_polls)
    if args.burst_nap >= 0:
        reft.reft_set_tunable("burst_nap", args.burst_nap)
    if args.burst_stage:
        reft.reft_set_tunable("burst_stage_bytes", args.burst_stage)
    if args.burst_wgs:
        reft.reft_set_tunable("burst_wgs_per_cu", args.burst_wgs)
    # s_snap / s_load carry the link-bound work (and, staged, the gather / scatter kernels);
    # s_copy / s_h2d carry the DMA transfers of the staged path; s_xor the HBM-bound XOR kernels.
    s_snap, s_xor, s_load = (torch.cuda.Stream() for _ in range(3))
    s_copy = torch.cuda.Stream() if save_staged and not args.one_stream_save else s_snap
    s_h2d = torch.cuda.Stream() if load_staged and args.two_stream_load else s_load
    snap_done_stream = s_copy
    enc_events, rec_events = [], []
    # The runtime maps streams to its few hardware queues in the order in which they first get
    # work; two streams on one queue run in turn.  Touch them in an order that keeps the two copy
    # directions and the XOR kernels apart.
    for st in (s_snap, s_copy, s_xor, s_load, s_h2d):
        with torch.cuda.stream(st):
            torch.zeros(1, device=dev)
    torch.cuda.synchronize()

    def save_phase(timed):
        """Parity encode, then the snapshot of the own shard, then the parity's snapshot.
        Returns the event after which the own shard's host copy is complete.  The encode runs
        before the copies start (16 ms during which the link idles): beside copy traffic that
        the runtime executes as kernels, as it does under rocprofv3, the write-burst kernel is
        several times slower, and a trainer would place the encode in a bubble anyway.
        --overlap-encode starts the own shard's snapshot first and the encode beside it."""
        if args.overlap_encode:
            reft.reft_snapshot_pack(plan, p_own, stag_save, host_snap, s_snap, s_copy)
            own_done = torch.cuda.Event()
            own_done.record(snap_done_stream)
        if timed:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(s_xor)
        reft.reft_parity_encode(plan, p_all, k, parity, s_xor)
        if timed:
            e1.record(s_xor)
            enc_events.append((e0, e1))
        s_snap.wait_stream(s_xor)
        if not args.overlap_encode:
            reft.reft_snapshot_pack(plan, p_own, stag_save, host_snap, s_snap, s_copy)
            own_done = torch.cuda.Event()
            own_done.record(snap_done_stream)
        reft.reft_snapshot_pack(pplan, p_par, stag_psave, host_par, s_snap, s_copy)
        return own_done

    def load_phase(timed, own_done):
        """Restore of the own shard (as soon as its snapshot is complete: it shares the link with
        the parity's snapshot, in the other direction), then the parity, then the decode."""
        first = s_h2d
        if not args.no_overlap_load:
            first.wait_event(own_done)
        else:
            first.wait_stream(snap_done_stream)
        reft.reft_restore(plan, host_snap, stag_load, p_fresh_own, s_h2d, s_load)
        first.wait_stream(snap_done_stream)             # the parity is complete on the host
        reft.reft_restore(pplan, host_par, stag_pload, p_par2, s_h2d, s_load)
        s_xor.wait_stream(s_load)
        if timed:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(s_xor)
        reft.reft_reconstruct_spans(plan, p_surv, k, lost, parity2, p_fresh_lost, s_xor)
        if timed:
            e1.record(s_xor)
            rec_events.append((e0, e1))
        # the next step's save may not overwrite what this step's load still reads
        s_snap.wait_stream(s_xor)
        s_snap.wait_stream(s_load)

    if args.has_demo:
        rec = has_demo(args, torch, reft, plan, pplan, L, k, p_own, p_all, p_par, parity, host_snap,
                       host_par, stag_save, stag_psave, s_snap, s_copy, s_xor)
        reft.reft_plan_destroy(plan)
        reft.reft_plan_destroy(pplan)
        print(json.dumps(rec), flush=True)
        return 0

    in_flight = []

    def step(timed=False):
        # Host-side pacing: at most two steps queued at once (a trainer takes one snapshot per
        # iteration; thousands of queued copies and events only slow the runtime down).
        if len(in_flight) >= 2:
            in_flight.pop(0).synchronize()
        load_phase(timed, save_phase(timed))
        done = torch.cuda.Event()
        done.record(s_xor)                      # the decode is the last thing a step does
        in_flight.append(done)

    if args.calibration_copy:
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(7)
        b = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(timed=True)
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t0
    ms_per_step = t_total / args.steps * 1e3
    value = 4 * L / (t_total / args.steps) / 1e9

    # ---- results are what they should be (device-side comparison with the source tensors) ------
    verified = all(torch.equal(a, b) for a, b in zip(fresh_own, shards[own])) and \
        all(torch.equal(a, b) for a, b in zip(fresh_lost, shards[lost]))
    if not verified:
        log("[bench] ERROR: restored or reconstructed tensors differ from the originals")

    enc_ms = sum(a.elapsed_time(b) for a, b in enc_events) / len(enc_events)
    rec_ms = sum(a.elapsed_time(b) for a, b in rec_events) / len(rec_events)
    enc_gbps = (k + 1) * L / (enc_ms * 1e-3) / 1e9
    rec_gbps = (k + 1) * L / (rec_ms * 1e-3) / 1e9

    # ---- each stage alone --------------------------------------------------------------------
    def pct(x, peak):
        return round(100.0 * x / peak, 1)

    def measure_stages():
        def timed_alone(fn, stream, reps=20, warm=3):
            """Median of `reps` timed repetitions after `warm` untimed ones."""
            for _ in range(warm):
                fn()
            torch.cuda.synchronize()
            ts = []
            for _ in range(reps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record(stream)
                fn()
                e1.record(stream)
                e1.synchronize()
                ts.append(e0.elapsed_time(e1) * 1e-3)
            ts.sort()
            return ts[len(ts) // 2]

        packed = torch.empty(L, dtype=torch.uint8, device=dev)
        t_pack = timed_alone(lambda: reft.reft_pack_device(plan, p_own, packed, s_xor), s_xor)
        t_unpack = timed_alone(lambda: reft.reft_unpack_device(plan, packed, p_fresh_own, s_xor), s_xor)
        t_enc = timed_alone(lambda: reft.reft_parity_encode(plan, p_all, k, parity, s_xor), s_xor)
        t_rec = timed_alone(lambda: reft.reft_reconstruct_spans(plan, p_surv, k, lost, parity2,
                                                                p_fresh_lost, s_xor), s_xor)
        del packed
        # the paper's rotated placement: all k members' units, then the decode of the lost member
        Lseg = reft.reft_segment_bytes(plan, k)
        units = [torch.empty(Lseg, dtype=torch.uint8, device=dev) for _ in range(k)]
        p_units = reft.ptr_array(units)

        def all_units():
            for i in range(k):
                reft.reft_parity_encode_rotated(plan, p_all, k, i, units[i], s_xor)
        t_rot = timed_alone(all_units, s_xor)
        t_rotdec = timed_alone(lambda: reft.reft_reconstruct_rotated(plan, p_all, p_units, k, lost,
                                                                     p_fresh_lost, s_xor), s_xor)
        rot_ok = all(torch.equal(a, b) for a, b in zip(fresh_lost, shards[lost]))
        del units

        def snap():
            s_snap.wait_stream(s_xor)
            reft.reft_snapshot_pack(plan, p_own, stag_save, host_snap, s_snap, s_copy)
            s_xor.wait_stream(snap_done_stream)
        def rest():
            s_h2d.wait_stream(s_xor)
            reft.reft_restore(plan, host_snap, stag_load, p_fresh_own, s_h2d, s_load)
            s_xor.wait_stream(s_load)
        t_snap = timed_alone(snap, s_xor, reps=5, warm=1)
        t_rest = timed_alone(rest, s_xor, reps=5, warm=1)

        stages = {
            "pack_kernel_GBps": round(2 * L / t_pack / 1e9, 1),
            "unpack_kernel_GBps": round(2 * L / t_unpack / 1e9, 1),
            "parity_encode_GBps": round((k + 1) * L / t_enc / 1e9, 1),
            "reconstruct_GBps": round((k + 1) * L / t_rec / 1e9, 1),
            "rotated_units_GBps": round(k * k * Lseg / t_rot / 1e9, 1),
            "rotated_decode_GBps": round(k * (k - 1) * Lseg / t_rotdec / 1e9, 1),
            "rotated_decode_verified": bool(rot_ok),
            "snapshot_d2h_GBps": round(L / t_snap / 1e9, 2),
            "restore_h2d_GBps": round(L / t_rest / 1e9, 2),
        }
        stages["pct_hbm_peak"] = {n: pct(stages[n], HBM_PEAK_GBPS) for n in
                                  ("pack_kernel_GBps", "unpack_kernel_GBps", "parity_encode_GBps",
                                   "reconstruct_GBps", "rotated_units_GBps", "rotated_decode_GBps")}
        stages["pct_link_peak"] = {n: pct(stages[n], LINK_PEAK_GBPS) for n in
                                   ("snapshot_d2h_GBps", "restore_h2d_GBps")}

        return stages

    stages = None if args.no_stages else measure_stages()

    # ---- concurrent training proxy: bf16 8192^3 GEMMs beside the save phase -------------------
    gemm = None
    if args.gemm_seconds >= 0:
        n = 8192
        A = torch.randn(n, n, device=dev, dtype=torch.bfloat16)
        B = torch.randn(n, n, device=dev, dtype=torch.bfloat16)
        C = torch.empty(n, n, device=dev, dtype=torch.bfloat16)
        cur = torch.cuda.current_stream()

        def gemms(count):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(cur)
            for _ in range(count):
                torch.matmul(A, B, out=C)
            e1.record(cur)
            return e0, e1

        e0, e1 = gemms(20)
        torch.cuda.synchronize()
        e0, e1 = gemms(50)
        torch.cuda.synchronize()
        t_one = e0.elapsed_time(e1) * 1e-3 / 50
        # the save phase alone
        torch.cuda.synchronize()
        ts0 = time.perf_counter()
        save_phase(False)
        torch.cuda.synchronize()
        t_save = time.perf_counter() - ts0
        ts0 = time.perf_counter()
        save_phase(False)
        torch.cuda.synchronize()
        t_save = min(t_save, time.perf_counter() - ts0)
        span = args.gemm_seconds if args.gemm_seconds > 0 else t_save
        count = max(10, int(span / t_one))
        e0, e1 = gemms(count)
        torch.cuda.synchronize()
        t_alone = e0.elapsed_time(e1) * 1e-3
        if args.snapshot_wgs:
            reft.reft_set_tunable("max_wgs", args.snapshot_wgs)
        torch.cuda.synchronize()
        ts0 = time.perf_counter()
        save_phase(False)
        e0, e1 = gemms(count)
        e1.synchronize()
        t_with = e0.elapsed_time(e1) * 1e-3
        torch.cuda.synchronize()
        t_save_with = time.perf_counter() - ts0
        reft.reft_set_tunable("max_wgs", 0)
        gemm = {
            "gemm": "bf16 8192x8192x8192 (torch.matmul as the load)",
            "gemms": count,
            "tflops_alone": round(2 * n ** 3 * count / t_alone / 1e12, 1),
            "t_alone_s": round(t_alone, 4),
            "t_with_snapshot_s": round(t_with, 4),
            "slowdown_pct": round(100.0 * (t_with - t_alone) / t_alone, 2),
            "save_phase_alone_s": round(t_save, 4),
            "save_phase_with_gemm_s": round(t_save_with, 4),
            "snapshot_wgs": args.snapshot_wgs,
        }
        del A, B, C

    # ---- bubble-aware scheduling of the save phase on a synthetic stage timeline ------------------
    has = None
    if save_staged and not args.no_has and args.gemm_seconds >= 0:
        has = has_demo(args, torch, reft, plan, pplan, L, k, p_own, p_all, p_par, parity, host_snap,
                       host_par, stag_save, stag_psave, s_snap, s_copy, s_xor, iterations=3)

    # ---- the CPU oracle on a bounded sample of the same workload --------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(wl, shards, own, lost, args.cpu_sample_mib << 20)

    record = {
        "metric": "snapshot+parity GB/s (% HBM/host-link peak); concurrent step slowdown %",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 2),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {
            "workload": f"config {wl.cfg}: {wl.description}",
            "k": k, "spans": T, "stream_bytes": L, "buckets": len(wl.bucket_nbytes),
            "step": "XOR parity, snapshot own shard + parity to pinned host, then "
                    "restore shard + parity from host and reconstruct the lost shard",
            "encode_beside_copies": bool(args.overlap_encode),
            "value_bytes_per_step": 4 * L,
            "save_path": args.save_path, "load_path": args.load_path,
            "staging_mib": args.staging_mib,
            "link_wgs": reft.reft_get_tunable("link_wgs"),
            "pct_link_peak_one_direction": pct(value, LINK_PEAK_GBPS),
            "note": "the own shard's restore overlaps the parity's snapshot: the link runs both "
                    "directions at once, so the step can exceed one direction's peak",
        },
        "verified": bool(verified),
        "roofline": {
            "kernel": f"k_gather_burst<{k}> (parity encode over {k} span tables)"
                      if reft.reft_get_tunable("burst") and k >= reft.reft_get_tunable("burst_min_rows")
                      else f"k_gather<{k}> (parity encode over {k} span tables)",
            "bound": "hbm",
            "achieved": round(enc_gbps, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(enc_gbps / HBM_PEAK_GBPS, 4),
            "traffic": measured_traffic(wl.cfg) if k == 8 else None,
            "bytes_per_launch": (k + 1) * L,
            "avg_launch_ms": round(enc_ms, 3),
            "reconstruct_achieved": round(rec_gbps, 1),
            "reconstruct_avg_launch_ms": round(rec_ms, 3),
        },
        "stages": stages,
        "gemm_proxy": gemm,
        "stage_timeline": has,
        "cpu_baseline": cpu,
    }
    reft.reft_plan_destroy(plan)
    reft.reft_plan_destroy(pplan)
    print(json.dumps(record), flush=True)
    return 0 if verified else 1


def has_demo(args, torch, reft, plan, pplan, L, k, p_own, p_all, p_par, parity, host_snap, host_par,
             stag_save, stag_psave, s_snap, s_copy, s_xor, iterations=5):
    """Hierarchical scheduling of one snapshot per iteration on a synthetic pipeline-stage timeline
    (Algorithm 1): each iteration is an idle bubble followed by a burst of bf16 GEMMs.

      none   no snapshot.
      naive  the whole save phase (encode, shard snapshot, parity snapshot; staged transport) is
             launched with the burst and runs beside it.
      has    layer 1: in the bubble, the parity encode and W_bubble = the buckets before the cut
             floor(n * t_bubble / t_ss) (SplitParameter), sent with the direct transport at full
             link rate; layer 2: the remaining buckets and the parity go out beside the burst with
             the staged transport (DMA copies, no kernels).

    t_ss = size / B_io (EstimateSnapshotTime) with B_io measured here; the bubble length is an
    input (the printed EstimateBubbleTime formula is not used)."""
    dev = torch.device("cuda:0")
    n = 8192
    A = torch.randn(n, n, device=dev, dtype=torch.bfloat16)
    B = torch.randn(n, n, device=dev, dtype=torch.bfloat16)
    C = torch.empty(n, n, device=dev, dtype=torch.bfloat16)
    s_gemm = torch.cuda.current_stream()
    nb = reft.reft_plan_num_buckets(plan)
    t_bubble = args.bubble_ms * 1e-3

    # B_io: the direct transport's rate on this machine
    reft.reft_snapshot_pack(plan, p_own, None, host_snap, s_snap, None)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    reft.reft_snapshot_pack(plan, p_own, None, host_snap, s_snap, None)
    torch.cuda.synchronize()
    b_io = L / (time.perf_counter() - t0)
    t_ss = L / b_io
    cut = reft.reft_plan_split(plan, 0.9 * t_bubble, t_ss)          # 10 % safety margin
    b_cut = reft.reft_plan_bucket_of(plan, cut)

    def burst():
        with torch.cuda.stream(s_gemm):
            for _ in range(args.burst_gemms):
                torch.matmul(A, B, out=C)
        ev = torch.cuda.Event()
        ev.record(s_gemm)
        return ev

    def save_all_beside_compute():
        reft.reft_parity_encode(plan, p_all, k, parity, s_xor)
        reft.reft_snapshot_pack(plan, p_own, stag_save, host_snap, s_snap, s_copy)
        s_snap.wait_stream(s_xor)
        reft.reft_snapshot_pack(pplan, p_par, stag_psave, host_par, s_snap, s_copy)

    def iteration(policy):
        t_start = time.perf_counter()
        if policy == "has":                      # layer 1: the bubble
            reft.reft_parity_encode(plan, p_all, k, parity, s_xor)
            reft.reft_snapshot_pack_range(plan, p_own, None, host_snap, 0, b_cut, s_snap, None)
        while time.perf_counter() - t_start < t_bubble:
            time.sleep(0.0005)
        done = burst()
        if policy == "naive":
            save_all_beside_compute()
        elif policy == "has":                    # layer 2: beside compute, copies only
            reft.reft_snapshot_pack_range(plan, p_own, stag_save, host_snap, b_cut, nb, s_snap, s_copy)
            s_snap.wait_stream(s_xor)
            reft.reft_snapshot_pack(pplan, p_par, stag_psave, host_par, s_snap, s_copy)
        done.synchronize()
        t_compute_done = time.perf_counter()
        torch.cuda.synchronize()                 # the snapshot must have landed before the next one
        return t_compute_done - t_start, time.perf_counter() - t_start

    out = {}
    for policy in ("none", "naive", "has", "none", "naive", "has"):
        iteration(policy)                        # warm-up
        its = [iteration(policy) for _ in range(iterations)]
        med = sorted(x[0] for x in its)[len(its) // 2]
        full = sorted(x[1] for x in its)[len(its) // 2]
        out.setdefault(policy, []).append((med, full))
    res = {p: (min(v[0][0], v[1][0]), min(v[0][1], v[1][1])) for p, v in out.items()}
    base = res["none"][0]
    return {
        "metric": "iteration time of a synthetic pipeline stage with one snapshot per iteration",
        "workload": f"config {args.config}",
        "bubble_ms": args.bubble_ms, "burst_gemms": args.burst_gemms,
        "B_io_GBps": round(b_io / 1e9, 2), "t_ss_ms": round(t_ss * 1e3, 1),
        "cut_bytes": cut, "cut_bucket": b_cut, "buckets": nb,
        "iteration_ms": {p: round(v[0] * 1e3, 2) for p, v in res.items()},
        "iteration_plus_snapshot_tail_ms": {p: round(v[1] * 1e3, 2) for p, v in res.items()},
        "overhead_pct": {p: round(100.0 * (v[0] - base) / base, 2) for p, v in res.items()},
    }


def measured_traffic(cfg: int):
    """HBM bytes per launch of the encode kernel from the committed rocprofv3 counter runs
    (FETCH_SIZE and WRITE_SIZE, each scaled by a copy of known size), or None if no such profile
    exists for this configuration."""
    path = os.path.join(ROOT, "profiles", f"config{cfg}_k_gather_burst8_hbm_traffic.txt")
    try:
        kv = {}
        for line in open(path):
            if "=" in line and line.split("=")[0].strip().startswith("traffic_"):
                key, _, val = line.partition("=")
                kv[key.strip()] = val.strip()
        if int(kv.get("traffic_config", -1)) == cfg:
            return int(kv["traffic_bytes"])
    except (OSError, ValueError, KeyError):
        pass
    return None


def cpu_baseline(wl, shards, own, lost, sample_bytes):
    """The oracle, as it stands, on the first spans of every shard (about ``sample_bytes`` each):
    pack the own shard, encode the parity, unpack the own shard, reconstruct and unpack the lost
    one.  Same numerator as the GPU figure (4 x sample stream bytes per pass)."""
    import numpy as np

    import oracle

    k = wl.k
    acc, nsp = 0, 0
    for s in wl.spans:
        if acc >= sample_bytes:
            break
        acc += s.nbytes
        nsp += 1
    Ls = acc
    sizes = [s.nbytes for s in wl.spans[:nsp]]
    cpu = [[oracle.as_bytes(t.cpu()) for t in sh[:nsp]] for sh in shards]
    buckets, left = [], Ls
    bsz = max(wl.bucket_nbytes)
    while left:
        buckets.append(min(left, bsz))
        left -= buckets[-1]

    def one_pass():
        t0 = time.perf_counter()
        streams = [oracle.pack_bucketed(cpu[own], buckets)]
        others = [oracle.pack(cpu[s]) for s in range(k) if s != own]   # peers' packed shards
        t_peers = time.perf_counter()
        all_streams = others[:own] + streams + others[own:]
        par = oracle.encode(all_streams)
        back = oracle.unpack(streams[0], sizes)
        rec = oracle.reconstruct([all_streams[s] for s in range(k) if s != lost], par)
        back_lost = oracle.unpack(rec, sizes)
        t1 = time.perf_counter()
        ok = all(np.array_equal(a, b) for a, b in zip(back_lost, cpu[lost])) and \
            all(np.array_equal(a, b) for a, b in zip(back, cpu[own]))
        return t1 - t0, ok

    out = {}
    threads_all = oracle.max_threads()
    for threads in (1, threads_all):
        oracle.set_threads(threads)
        t, ok = one_pass()
        out[threads] = (t, ok)
    oracle.set_threads(1)
    t_all, ok_all = out[threads_all]
    t_one, ok_one = out[1]
    return {
        "value": round(4 * Ls / t_all / 1e9, 3),
        "unit": "GB/s",
        "cores": threads_all,
        "kind": "oracle",
        "sample": f"first {nsp} spans of each of the {k} shards ({Ls} bytes per shard); one pass = "
                  f"pack own + pack peers + encode + unpack + reconstruct + unpack, {t_all:.2f} s",
        "single_thread_value": round(4 * Ls / t_one / 1e9, 3),
        "single_thread_seconds": round(t_one, 2),
        "verified": bool(ok_all and ok_one),
    }


if __name__ == "__main__":
    sys.exit(main())
