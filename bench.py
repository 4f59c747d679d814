#!/usr/bin/env python3
"""Benchmark of the in-memory checkpointing hot path on one MI355X.

One *step* is one pass of the whole path over one rank-shaped synthetic state, inputs resident in
HBM before the clock starts:

  save   reft_parity_encode   k shards    -> parity (device)                  (k-way XOR, in place)
         reft_snapshot_pack   own shard   -> pinned host   (staged transport: DMA copies straight
                                                            from the tensors, gather kernel only
                                                            for runs of small tensors)
         reft_snapshot_pack   parity      -> pinned host
  load   reft_restore         host shard  -> fresh tensors  (staged transport as well)
         reft_restore         host parity -> device
         reft_reconstruct_spans  k-1 survivors + parity -> lost shard's tensors (k-way XOR)

Consecutive steps are software-pipelined the way a trainer that checkpoints every iteration and a
recovery that loads the last complete checkpoint would share the machine: the host link carries
snapshots (device to host) and restores (host to device) at the same time.  Per step, in order on
the save stream: [encode of step n, decode of step n-2] (the XOR window: it opens when the previous
step's copies have ended, so nothing runs beside the two HBM-bound kernels), snapshot of the
shard, snapshot of the parity; on the load stream:
restore of the shard (beside the parity's snapshot), restore of the parity (beside the next step's
shard snapshot).  Every dependency is an event: a host buffer is overwritten only after its
restore has read it, the parity is restored only after the decode that read the previous one.
The timed region holds exactly K encodes, 2 K snapshots, 2 K restores and K decodes; the
pipeline fills and drains inside it.  ``--serial`` runs the steps one after the other instead.

``value`` is the step's checkpoint traffic, 4*L bytes (shard + parity saved to host, shard + parity
loaded back), divided by the step time: the path is bound by the host link, which is why the
HBM-bound kernels are reported separately under ``stages`` and ``roofline``.

The record's headline is the configuration the metric's "concurrent step slowdown" is defined on
(3: 34B-shaped, 8 x 15 GB); ``per_config`` holds a shorter run of the other Llama-shaped
configurations.  The last line printed is the JSON record.  ``python bench.py --help`` lists the
options.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0           # MI355X HBM3E, published
LINK_PEAK_GBPS = 63.0            # PCIe Gen5 x16, one direction: 32 GT/s * 16 * 128/130 / 8
LINK_DUPLEX_PEAK_GBPS = 2 * LINK_PEAK_GBPS


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def pct(x, peak):
    return round(100.0 * x / peak, 1)


def parse_args():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawTextHelpFormatter)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3, help="workload configuration 0..4 (default 3)")
    ap.add_argument("--per-config", type=str, default="1,2,4",
                    help="configurations that get a shorter run of their own under per_config "
                         "(comma separated; '' = none)")
    ap.add_argument("--per-config-steps", type=int, default=8)
    ap.add_argument("--serial", action="store_true",
                    help="no pipelining across steps: a step's save starts when the previous "
                         "step's load has ended")
    ap.add_argument("--queue-depth", type=int, default=1, choices=[1, 2, 3],
                    help="before queuing a step the host waits until the parity snapshot or the "
                         "shard restore of the step this many steps back has ended, whichever "
                         "comes first (default 1).  The runtime picks a copy engine for a stream "
                         "when its copies are queued: with the link idle at that moment the two "
                         "directions can land on one engine and run one after the other, and with "
                         "two or three steps' copies queued ahead (some 4000 hipMemcpyAsync calls) "
                         "the choice climbs to engines that move host traffic at a quarter of the "
                         "rate")
    ap.add_argument("--settle-seconds", type=float, default=6.0,
                    help="pause before the steps of each further configuration (--per-config): for "
                         "a few seconds after a configuration's 100-170 GB of device memory have "
                         "been freed, host-to-device copies run at half rate beside a device-to-"
                         "host copy (437 instead of 222 ms for the first shard restore; with the "
                         "pause it does not happen), presumably while the driver clears the freed "
                         "memory")
    ap.add_argument("--pace-on", choices=["first", "parity"], default="first",
                    help="first (default): queue a step when the first of the two copy streams has "
                         "finished the previous one.  parity: the earlier rule, kept to show what "
                         "it costs (wait for the previous parity snapshot, no engine re-choice): "
                         "the second step after a start runs its two directions one after the "
                         "other")
    ap.add_argument("--trace-phases", action="store_true",
                    help="log when each phase of each timed step began and ended (HIP events)")
    ap.add_argument("--gemm-seconds", type=float, default=0.0,
                    help="length of the bf16 GEMM proxy loop for the slowdown figure "
                         "(0 = as long as one save phase; negative = skip)")
    ap.add_argument("--snapshot-wgs", type=int, default=0,
                    help="cap on workgroups of the snapshot kernels while the GEMM proxy runs")
    ap.add_argument("--save-path", choices=["direct", "staged"], default="staged",
                    help="snapshot transport. staged: hipMemcpyAsync on the DMA engines (what runs "
                         "beside training); direct: the gather kernel stores to pinned host memory")
    ap.add_argument("--load-path", choices=["direct", "staged"], default="staged",
                    help="restore transport. staged (default): runtime copies, which share the link "
                         "well with a snapshot going the other way; direct: the scatter kernel "
                         "reads pinned host memory itself (fastest when nothing else runs)")
    ap.add_argument("--dma-streams", type=int, default=0, choices=[0, 1, 2],
                    help="staged transport: 2 = piece copies alternate with a helper stream "
                         "(0 = library default)")
    ap.add_argument("--staging-mib", type=int, default=1024,
                    help="size of each staging ring in MiB (split into bucket-sized slots)")
    ap.add_argument("--link-wgs", type=int, default=0,
                    help="cap on workgroups of the link-bound kernels (0 = library default)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain device-to-device copy of 1 GiB (torch), the kernel of "
                         "known size that scales the rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
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
    ap.add_argument("--stage-reps", type=int, default=20)
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
    return ap.parse_args()


class Bench:
    """One configuration resident on the GPU: state, plans, buffers, streams, and the step."""

    def __init__(self, args, cfg, torch, reft, pinned, streams):
        from workload import fill_shard, make_workload, span_nbytes

        self.args, self.torch, self.reft = args, torch, reft
        self.dev = dev = torch.device("cuda:0")
        # two streams carry a step: s_save the XOR kernels and the snapshots, s_load the restores
        self.s_save, self.s_load = streams
        self.wl = wl = make_workload(cfg)
        self.k, self.L, self.T = wl.k, wl.L, len(wl.spans)
        k, L = self.k, self.L
        self.lost = wl.lost
        self.own = (wl.lost + 1) % k
        log(f"[bench] config {wl.cfg}: {wl.description}; k={k} T={self.T} L={L} "
            f"buckets={len(wl.bucket_nbytes)} lost={self.lost} own={self.own}")
        t0 = time.time()
        self.shards = [fill_shard(wl, s, dev) for s in range(k)]
        torch.cuda.synchronize()
        log(f"[bench] generated {k * L / 1e9:.1f} GB of state in {time.time() - t0:.1f} s")

        self.plan = reft.reft_plan_create(span_nbytes(wl), wl.bucket_nbytes)
        bucket = reft.reft_plan_max_bucket_bytes(self.plan)
        self.pplan = reft.reft_plan_create([L], None, bucket)      # the parity as a 1-span shard
        self.save_staged = args.save_path == "staged"
        self.load_staged = args.load_path == "staged"

        def ring(p, use):
            if not use:
                return None
            slot = reft.reft_plan_staging_slot_bytes(p)
            nslots = max(2, min(64, (args.staging_mib << 20) // slot))
            return torch.empty(nslots * slot, dtype=torch.uint8, device=dev)
        # the staged transport needs its ring only for runs of small pieces
        self.gathers, self.copies = reft.reft_plan_staged_work(self.plan)
        self.stag_save = ring(self.plan, self.save_staged)
        self.stag_psave = ring(self.pplan, self.save_staged)
        self.stag_load = ring(self.plan, self.load_staged)
        self.stag_pload = ring(self.pplan, self.load_staged)
        self.host_snap, self.host_par = pinned[0][:L], pinned[1][:L]
        self.parity = torch.empty(L, dtype=torch.uint8, device=dev)
        self.parity2 = torch.empty(L, dtype=torch.uint8, device=dev)
        self.fresh_own = [torch.empty_like(t) for t in self.shards[self.own]]
        self.fresh_lost = [torch.empty_like(t) for t in self.shards[self.lost]]

        sh = self.shards
        self.p_own = reft.ptr_array(sh[self.own])
        self.p_all = reft.ptr_array([t for s in sh for t in s])
        self.p_surv = reft.ptr_array([None if s == self.lost else t for s, x in enumerate(sh) for t in x])
        self.p_fresh_own = reft.ptr_array(self.fresh_own)
        self.p_fresh_lost = reft.ptr_array(self.fresh_lost)
        self.p_par = reft.ptr_array([self.parity])
        self.p_par2 = reft.ptr_array([self.parity2])

        # A staged snapshot that gathers runs of small pieces puts those kernels on a stream of
        # their own (s_pack); the Llama-shaped configurations have no such runs, and one stream
        # serves as pack_stream and copy_stream (a hardware queue less).
        self.s_pack = torch.cuda.Stream() if (self.save_staged and self.gathers) else self.s_save
        self.enc_events, self.dec_events = [], []
        self.phases, self.tracing, self.step_marks = [], False, []
        self.reset_pipeline()

    # ---- the step ---------------------------------------------------------------------------------
    # Buffers and who touches them: parity (encode writes, parity snapshot reads; both on s_save),
    # host_snap (shard snapshot writes, shard restore reads), host_par (parity snapshot writes,
    # parity restore reads), parity2 (parity restore writes, decode reads).  ev[name][n] is recorded
    # behind the named operation of step n.
    def reset_pipeline(self):
        self.n = 0
        self.ev = {name: {} for name in ("shard_saved", "par_saved", "shard_restored",
                                         "par_restored", "decoded", "window_closed", "load_turn")}

    def _mark(self, name, n, stream):
        e = self.torch.cuda.Event()
        e.record(stream)
        self.ev[name][n] = e
        self.ev[name].pop(n - 4, None)

    def _wait(self, stream, name, n):
        e = self.ev[name].get(n)
        if e is not None:
            stream.wait_event(e)

    def _phase(self, name, n, stream, fn):
        """Run fn; with --trace-phases, bracket it with timing events on its stream."""
        if not (self.args.trace_phases and self.tracing):
            fn()
            return
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        fn()
        e1.record(stream)
        self.phases.append((name, n, e0, e1))

    def _timed(self, timed, store, fn):
        if not timed:
            fn()
            return
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(self.s_save)
        fn()
        e1.record(self.s_save)
        store.append((e0, e1))

    def _encode(self, n, timed):
        self._timed(timed, self.enc_events, lambda: self.reft.reft_parity_encode(
            self.plan, self.p_all, self.k, self.parity, self.s_save))

    def _decode(self, n, timed):
        self._wait(self.s_save, "par_restored", n)
        self._timed(timed, self.dec_events, lambda: self.reft.reft_reconstruct_spans(
            self.plan, self.p_surv, self.k, self.lost, self.parity2, self.p_fresh_lost, self.s_save))
        self._mark("decoded", n, self.s_save)

    def _snapshot_shard(self, n):
        self._wait(self.s_save, "shard_restored", n - 1)          # host_snap has been read
        if self.s_pack is not self.s_save:
            self.s_pack.wait_stream(self.s_save)
        self._phase("snapshot_shard", n, self.s_save, lambda: self.reft.reft_snapshot_pack(
            self.plan, self.p_own, self.stag_save, self.host_snap, self.s_pack, self.s_save))
        self._mark("shard_saved", n, self.s_save)

    def _snapshot_parity(self, n):
        self._wait(self.s_save, "par_restored", n - 1)            # host_par has been read
        if self.s_pack is not self.s_save:
            self.s_pack.wait_stream(self.s_save)                  # the encode produced the parity
        self._phase("snapshot_parity", n, self.s_save, lambda: self.reft.reft_snapshot_pack(
            self.pplan, self.p_par, self.stag_psave, self.host_par, self.s_pack, self.s_save))
        self._mark("par_saved", n, self.s_save)
        if self.tracing:                                          # one timing mark per timed step
            e = self.torch.cuda.Event(enable_timing=True)
            e.record(self.s_save)
            self.step_marks.append(e)

    def _restore_shard(self, n):
        self._wait(self.s_load, "shard_saved", n)
        self._phase("restore_shard", n, self.s_load, lambda: self.reft.reft_restore(
            self.plan, self.host_snap, self.stag_load, self.p_fresh_own, self.s_load, self.s_load))
        self._mark("shard_restored", n, self.s_load)

    def _restore_parity(self, n):
        self._wait(self.s_load, "par_saved", n)
        self._wait(self.s_load, "decoded", n - 1)                 # parity2 has been read
        self._phase("restore_parity", n, self.s_load, lambda: self.reft.reft_restore(
            self.pplan, self.host_par, self.stag_pload, self.p_par2, self.s_load, self.s_load))
        self._mark("par_restored", n, self.s_load)

    def _pace(self, n):
        """Host-side pacing: queue step n once one of the two copy streams has finished step
        n - queue_depth and the other is still busy with it.

        Why this moment (read from the runtime's own log, AMD_LOG_LEVEL=4): a stream's copies go to
        the lowest-numbered copy engine that has nothing pending at the time the stream chooses, and
        a stream chooses again only when it waits for another stream right behind its copies.  If
        both streams are idle when a step is queued (which happens once, in the second step after
        a start, where the parity snapshot outlasts the shard restore), the load stream takes the
        save stream's engine, the save stream keeps it, and each phase's piece copies run only
        after the other direction's 15 GB copy (530 ms instead of 300, twice).  With one of the two
        still busy the choices never collide.  Queuing earlier is no remedy: with more copies
        pending the choice climbs to engines 0x10 and 0x20, which moved host traffic at 13 and
        24 GB/s instead of 56."""
        a = self.ev["par_saved"].get(n - self.args.queue_depth)
        b = self.ev["shard_restored"].get(n - self.args.queue_depth)
        if a is None or b is None:
            return
        if self.args.pace_on == "parity":
            a.synchronize()
            return
        while not (a.query() or b.query()):
            time.sleep(100e-6)

    def _rechoose_engine(self, n):
        """Make the save stream wait, through the load stream, for its own shard snapshot.

        The wait orders nothing new; it is there because a stream keeps its copy engine until a
        wait for another stream has come true (see _pace).  Step 0 has no such wait on the save
        stream, so in step 1 the save stream would still sit on the engine that the load stream,
        choosing again with everything idle, has just taken."""
        if self.args.pace_on == "parity":
            return
        self._wait(self.s_load, "shard_saved", n)
        self._mark("load_turn", n, self.s_load)
        self._wait(self.s_save, "load_turn", n)

    def step(self, timed=False):
        n = self.n
        self._pace(n)
        # The XOR window opens when the previous step's shard restore has ended (the next snapshot
        # needs its host buffer read anyway): DMA writes trickling into HBM beside the XOR kernels
        # cost them 5 % (measured), and nothing else is in flight at this point.
        self._wait(self.s_save, "shard_restored", n - 1)
        self._encode(n, timed)
        if self.args.serial:
            self._snapshot_shard(n)
            self._snapshot_parity(n)
            self._restore_shard(n)                  # beside the parity's snapshot
            self._restore_parity(n)
            self._decode(n, timed)
        else:
            if n >= 2:
                self._decode(n - 2, timed)          # the XOR window: encode(n), decode(n-2)
            if n >= 1:
                # beside this step's shard snapshot, and behind the window also in the first steps,
                # where no decode holds it back yet
                self._mark("window_closed", n, self.s_save)
                self._wait(self.s_load, "window_closed", n)
                self._restore_parity(n - 1)
            self._snapshot_shard(n)
            self._rechoose_engine(n)
            self._snapshot_parity(n)
            self._restore_shard(n)                  # beside this step's parity snapshot
        self.n = n + 1

    def drain(self, timed=False):
        """Queue what the pipeline still owes after the last step."""
        n = self.n
        if not self.args.serial and n >= 1:
            self._wait(self.s_save, "shard_restored", n - 1)      # the last window, as in step()
            if n >= 2:
                self._decode(n - 2, timed)
            self._restore_parity(n - 1)
            self._decode(n - 1, timed)
        self.reset_pipeline()

    def save_phase(self):
        """The save half alone (what runs beside training): encode, shard snapshot, parity snapshot."""
        self._encode(0, False)
        self._snapshot_shard(0)
        self._snapshot_parity(0)
        self.reset_pipeline()

    def verified(self):
        torch = self.torch
        return all(torch.equal(a, b) for a, b in zip(self.fresh_own, self.shards[self.own])) and \
            all(torch.equal(a, b) for a, b in zip(self.fresh_lost, self.shards[self.lost]))

    def close(self):
        self.reft.reft_plan_destroy(self.plan)
        self.reft.reft_plan_destroy(self.pplan)


# --------------------------------------------------------------------------------------------------
# measurements on one configuration
# --------------------------------------------------------------------------------------------------
def run_steps(b, steps, warmup):
    torch = b.torch
    for _ in range(warmup):
        b.step()
    b.drain()
    torch.cuda.synchronize()
    # poison the outputs so that the check below sees this run's results
    for t in b.fresh_own + b.fresh_lost:
        t.view(torch.uint8).fill_(0x5A)
    torch.cuda.synchronize()
    b.enc_events.clear()
    b.dec_events.clear()
    b.step_marks.clear()
    b.tracing = True
    base = torch.cuda.Event(enable_timing=True)
    base.record(b.s_save)
    t0 = time.perf_counter()
    for _ in range(steps):
        b.step(timed=True)
    b.drain(timed=True)
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t0
    b.tracing = False
    if b.args.trace_phases:
        rows = [(base.elapsed_time(e0), base.elapsed_time(e1), name, n) for name, n, e0, e1 in b.phases]
        rows += [(base.elapsed_time(x), base.elapsed_time(y), "encode", i) for i, (x, y) in enumerate(b.enc_events)]
        rows += [(base.elapsed_time(x), base.elapsed_time(y), "decode", i) for i, (x, y) in enumerate(b.dec_events)]
        for t_a, t_b, name, n in sorted(rows):
            log(f"[phase] {t_a:9.1f} .. {t_b:9.1f} ms  ({t_b - t_a:7.1f})  {name}({n})")
        b.phases.clear()
    ok = b.verified()
    if not ok:
        log("[bench] ERROR: restored or reconstructed tensors differ from the originals")
    enc_ms = sum(x.elapsed_time(y) for x, y in b.enc_events) / len(b.enc_events)
    dec_ms = sum(x.elapsed_time(y) for x, y in b.dec_events) / len(b.dec_events)
    assert len(b.enc_events) == steps and len(b.dec_events) == steps
    # steady state: the median interval between the ends of consecutive steps' parity snapshots,
    # the first three steps (pipeline fill, start-up transient) left out
    gaps = sorted(x.elapsed_time(y) for x, y in zip(b.step_marks[3:], b.step_marks[4:]))
    steady = gaps[len(gaps) // 2] * 1e-3 if gaps else None
    return t_total / steps, enc_ms, dec_ms, ok, steady


def measure_stages(b, reps):
    torch, reft = b.torch, b.reft
    k, L, dev, plan, pplan = b.k, b.L, b.dev, b.plan, b.pplan
    s = b.s_save

    def timed_alone(fn, stream, reps=reps, warm=3):
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
    t_pack = timed_alone(lambda: reft.reft_pack_device(plan, b.p_own, packed, s), s)
    t_unpack = timed_alone(lambda: reft.reft_unpack_device(plan, packed, b.p_fresh_own, s), s)
    # the 1:1 ceiling the two are held against: the same kernel as a plain copy of one span of L
    # bytes (16-byte vectors, nothing ragged), and the runtime's own device copy for scale
    t_copy = timed_alone(lambda: reft.reft_pack_device(pplan, b.p_par, packed, s), s)
    with torch.cuda.stream(s):
        t_blit = timed_alone(lambda: packed.copy_(b.parity), s, reps=min(reps, 7))
    t_enc = timed_alone(lambda: reft.reft_parity_encode(plan, b.p_all, k, b.parity, s), s)
    burst = dict(zip(("rounds_met", "rounds_timed_out", "rounds_not_waited", "group_completions"),
                     reft.reft_plan_burst_stats(plan)))
    t_rec = timed_alone(lambda: reft.reft_reconstruct_spans(plan, b.p_surv, k, b.lost, b.parity2,
                                                            b.p_fresh_lost, s), s)
    # pack + encode in one pass (the own shard is read once for both)
    t_fused = timed_alone(lambda: reft.reft_parity_encode_pack(plan, b.p_all, k, b.own, b.parity,
                                                               packed, s), s)
    fused_ok = bool(torch.equal(packed, torch.cat([t.reshape(-1).view(torch.uint8) for t in b.shards[b.own]])))
    del packed
    # the paper's rotated placement: all k members' units, then the decode of the lost member
    Lseg = reft.reft_segment_bytes(plan, k)
    units = [torch.empty(Lseg, dtype=torch.uint8, device=dev) for _ in range(k)]
    p_units = reft.ptr_array(units)

    def all_units():
        for i in range(k):
            reft.reft_parity_encode_rotated(plan, b.p_all, k, i, units[i], s)
    t_rot = timed_alone(all_units, s, reps=min(reps, 10))
    t_rotdec = timed_alone(lambda: reft.reft_reconstruct_rotated(plan, b.p_all, p_units, k, b.lost,
                                                                 b.p_fresh_lost, s), s, reps=min(reps, 10))
    rot_ok = all(torch.equal(x, y) for x, y in zip(b.fresh_lost, b.shards[b.lost]))
    del units

    def snap():
        reft.reft_snapshot_pack(plan, b.p_own, b.stag_save, b.host_snap, b.s_pack, s)
        if b.s_pack is not s:
            s.wait_stream(b.s_pack)

    def rest():
        reft.reft_restore(plan, b.host_snap, b.stag_load, b.p_fresh_own, s, s)

    def both():                                     # the two directions of the link at once
        b.s_load.wait_stream(s)                     # the restore starts with the timed region
        reft.reft_snapshot_pack(pplan, b.p_par, b.stag_psave, b.host_par, b.s_pack, s)
        reft.reft_restore(plan, b.host_snap, b.stag_load, b.p_fresh_own, b.s_load, b.s_load)
        s.wait_stream(b.s_load)
    t_snap = timed_alone(snap, s, reps=5, warm=1)
    t_rest = timed_alone(rest, s, reps=5, warm=1)
    t_both = timed_alone(both, s, reps=5, warm=1)

    stages = {
        "pack_kernel_GBps": round(2 * L / t_pack / 1e9, 1),
        "unpack_kernel_GBps": round(2 * L / t_unpack / 1e9, 1),
        "copy_ceiling_GBps": round(2 * L / t_copy / 1e9, 1),
        "runtime_copy_GBps": round(2 * L / t_blit / 1e9, 1),
        "parity_encode_GBps": round((k + 1) * L / t_enc / 1e9, 1),
        "reconstruct_GBps": round((k + 1) * L / t_rec / 1e9, 1),
        "fused_pack_encode_GBps": round((k + 2) * L / t_fused / 1e9, 1),
        "fused_pack_encode": {"ms": round(t_fused * 1e3, 3), "encode_then_pack_ms": round((t_enc + t_pack) * 1e3, 3),
                              "hbm_bytes": (k + 2) * L, "encode_then_pack_hbm_bytes": (k + 3) * L,
                              "packed_copy_verified": fused_ok},
        "rotated_units_GBps": round(k * k * Lseg / t_rot / 1e9, 1),
        "rotated_decode_GBps": round(k * (k - 1) * Lseg / t_rotdec / 1e9, 1),
        "rotated_decode_verified": bool(rot_ok),
        "snapshot_d2h_GBps": round(L / t_snap / 1e9, 2),
        "restore_h2d_GBps": round(L / t_rest / 1e9, 2),
        "duplex_GBps": round(2 * L / t_both / 1e9, 2),
        "encode_burst_rounds": burst,
        "note": "copy_ceiling = the gather kernel as a plain copy of L bytes in one span (the 1:1 "
                "streaming ceiling of this part for hand-written 16-byte-vector code); duplex = one "
                "snapshot and one restore of L bytes each at the same time, both directions summed",
    }
    stages["pct_hbm_peak"] = {n: pct(stages[n], HBM_PEAK_GBPS) for n in
                              ("pack_kernel_GBps", "unpack_kernel_GBps", "copy_ceiling_GBps",
                               "parity_encode_GBps", "reconstruct_GBps", "fused_pack_encode_GBps",
                               "rotated_units_GBps", "rotated_decode_GBps")}
    stages["pct_link_peak"] = {"snapshot_d2h_GBps": pct(stages["snapshot_d2h_GBps"], LINK_PEAK_GBPS),
                               "restore_h2d_GBps": pct(stages["restore_h2d_GBps"], LINK_PEAK_GBPS),
                               "duplex_GBps": pct(stages["duplex_GBps"], LINK_DUPLEX_PEAK_GBPS)}
    return stages


def gemm_proxy(b):
    """bf16 8192^3 GEMMs on the current stream, alone and beside one save phase."""
    torch, reft, args = b.torch, b.reft, b.args
    n = 8192
    A = torch.randn(n, n, device=b.dev, dtype=torch.bfloat16)
    B = torch.randn(n, n, device=b.dev, dtype=torch.bfloat16)
    C = torch.empty(n, n, device=b.dev, dtype=torch.bfloat16)
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
    t_save = 1e9
    for _ in range(2):                                   # the save phase alone
        torch.cuda.synchronize()
        ts0 = time.perf_counter()
        b.save_phase()
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
    b.save_phase()
    e0, e1 = gemms(count)
    e1.synchronize()
    t_with = e0.elapsed_time(e1) * 1e-3
    torch.cuda.synchronize()
    t_save_with = time.perf_counter() - ts0
    reft.reft_set_tunable("max_wgs", 0)
    return {
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


def run_config(args, cfg, torch, reft, pinned, streams, primary):
    """All measurements of one configuration; returns its part of the record."""
    b = Bench(args, cfg, torch, reft, pinned, streams)
    k, L = b.k, b.L
    try:
        if args.has_demo:
            return has_demo(b)
        if args.calibration_copy and primary:
            x = torch.empty(1 << 30, dtype=torch.uint8, device=b.dev).fill_(7)
            y = torch.empty(1 << 30, dtype=torch.uint8, device=b.dev)
            y.copy_(x)
            torch.cuda.synchronize()
            del x, y
        steps = args.steps if primary else args.per_config_steps
        warmup = args.warmup if primary else 1
        if not primary:
            time.sleep(args.settle_seconds)     # see --settle-seconds
        t_step, enc_ms, dec_ms, ok, steady = run_steps(b, steps, warmup)
        value = 4 * L / t_step / 1e9
        enc_gbps = (k + 1) * L / (enc_ms * 1e-3) / 1e9
        dec_gbps = (k + 1) * L / (dec_ms * 1e-3) / 1e9
        burst_on = reft.reft_get_tunable("burst") and k >= reft.reft_get_tunable("burst_min_rows")
        traffic, source = measured_traffic(b.wl.cfg)
        out = {
            "workload": f"config {b.wl.cfg}: {b.wl.description}",
            "k": k, "spans": b.T, "stream_bytes": L, "buckets": len(b.wl.bucket_nbytes),
            "staged_snapshot": {"gather_launches": b.gathers, "copies": b.copies},
            "steps": steps, "warmup": warmup,
            "ms_per_step": round(t_step * 1e3, 2),
            "value_GBps": round(value, 2),
            "pct_link_duplex_peak": pct(value, LINK_DUPLEX_PEAK_GBPS),
            "steady_state": None if steady is None else {
                "ms_per_step": round(steady * 1e3, 2),
                "GBps": round(4 * L / steady / 1e9, 2),
                "pct_link_duplex_peak": pct(4 * L / steady / 1e9, LINK_DUPLEX_PEAK_GBPS),
                "note": "median interval between consecutive steps inside the timed region (HIP "
                        "events), fill, drain and the first three steps left out; context for "
                        "value, which is the whole timed region"},
            "verified": bool(ok),
            "roofline": {
                "kernel": (f"k_gather_burst<{k}>" if burst_on else f"k_gather<{k}>") +
                          f" (parity encode over {k} span tables)",
                "bound": "hbm",
                "achieved": round(enc_gbps, 1),
                "peak": HBM_PEAK_GBPS,
                "unit": "GB/s",
                "frac": round(enc_gbps / HBM_PEAK_GBPS, 4),
                "traffic": traffic,
                "traffic_source": source,
                "bytes_per_launch": (k + 1) * L,
                "avg_launch_ms": round(enc_ms, 3),
                "reconstruct_achieved": round(dec_gbps, 1),
                "reconstruct_frac": round(dec_gbps / HBM_PEAK_GBPS, 4),
                "reconstruct_avg_launch_ms": round(dec_ms, 3),
            },
        }
        if not args.no_stages:
            out["stages"] = measure_stages(b, args.stage_reps)
        if args.gemm_seconds >= 0:
            out["gemm_proxy"] = gemm_proxy(b)
        if primary and b.save_staged and not args.no_has and args.gemm_seconds >= 0:
            out["stage_timeline"] = has_demo(b, iterations=3)
        if primary and not args.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline(b.wl, b.shards, b.own, b.lost, args.cpu_sample_mib << 20)
        return out
    finally:
        b.close()
        del b
        gc.collect()
        torch.cuda.empty_cache()


def main() -> int:
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU (the simulated node's k shards live in one "
              "GPU's HBM); --gpus N with N > 1 is not supported.", file=sys.stderr)
        return 2

    import torch

    import paper_2310_12670_amd as reft
    from workload import make_workload

    assert torch.cuda.is_available(), "bench.py needs the GPU (there is no CPU path)"
    torch.cuda.set_device(torch.device("cuda:0"))
    # The step's two streams are made before anything else that makes streams: the runtime deals
    # streams onto its few hardware queues (4 per process here) as they are created, and two
    # streams on one queue take turns, which would cost the step its full-duplex use of the link.
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    for st in streams:
        with torch.cuda.stream(st):
            torch.zeros(1, device="cuda:0")
    torch.cuda.synchronize()
    others = [] if args.has_demo else \
        [int(c) for c in args.per_config.split(",") if c.strip() and int(c) != args.config]

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

    # one pair of pinned host buffers serves every configuration (the box pins a limited amount)
    t0 = time.time()
    Lmax = max(make_workload(c).L for c in [args.config] + others)
    pinned = [torch.empty(Lmax, dtype=torch.uint8, pin_memory=True) for _ in range(2)]
    log(f"[bench] pinned {2 * Lmax / 1e9:.1f} GB of host memory in {time.time() - t0:.1f} s")

    main_rec = run_config(args, args.config, torch, reft, pinned, streams, primary=True)
    if args.has_demo:
        print(json.dumps(main_rec), flush=True)
        return 0
    per = {}
    for c in others:
        per[f"config{c}"] = run_config(args, c, torch, reft, pinned, streams, primary=False)

    value = main_rec["value_GBps"]
    record = {
        "metric": "snapshot+parity GB/s (% HBM/host-link peak); concurrent step slowdown %",
        "value": value,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": main_rec["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {
            "workload": main_rec["workload"],
            "k": main_rec["k"], "spans": main_rec["spans"], "stream_bytes": main_rec["stream_bytes"],
            "buckets": main_rec["buckets"],
            "step": "XOR parity, snapshot own shard + parity to pinned host, restore shard + parity "
                    "from host and reconstruct the lost shard; consecutive steps " +
                    ("run one after the other" if args.serial else
                     "are pipelined so that snapshots and restores share the link, full duplex; the "
                     "XOR kernels run with the link idle"),
            "schedule": "serial" if args.serial else "pipelined",
            "value_bytes_per_step": 4 * main_rec["stream_bytes"],
            "save_path": args.save_path, "load_path": args.load_path,
            "staged_snapshot": main_rec["staged_snapshot"],
            "dma_streams": reft.reft_get_tunable("dma_streams"),
            "pct_link_duplex_peak": main_rec["pct_link_duplex_peak"],
            "steady_state": main_rec["steady_state"],
            "link_peak_GBps": {"one_direction": LINK_PEAK_GBPS, "duplex": LINK_DUPLEX_PEAK_GBPS},
            "note": "value counts bytes in both directions of the host link, so it is held against "
                    "the duplex peak; each direction alone is under stages.pct_link_peak",
        },
        "verified": bool(main_rec["verified"] and all(r["verified"] for r in per.values())),
        "roofline": main_rec["roofline"],
        "stages": main_rec.get("stages"),
        "gemm_proxy": main_rec.get("gemm_proxy"),
        "stage_timeline": main_rec.get("stage_timeline"),
        "cpu_baseline": main_rec.get("cpu_baseline"),
        "per_config": per,
    }
    print(json.dumps(record), flush=True)
    return 0 if record["verified"] else 1


def has_demo(b, iterations=5):
    """Hierarchical scheduling of one snapshot per iteration on a synthetic pipeline-stage timeline
    (Algorithm 1): each iteration is an idle bubble followed by a burst of bf16 GEMMs.

      none   no snapshot.
      naive  the whole save phase (encode, shard snapshot, parity snapshot; staged transport) is
             launched with the burst and runs beside it.
      has    layer 1: in the bubble, the parity encode and W_bubble = the buckets before the cut
             floor(n * t_bubble / t_ss) (SplitParameter), sent with the direct transport at full
             link rate; layer 2: the remaining buckets and the parity go out beside the burst with
             the staged transport (DMA copies, no kernels).
      fused  in the bubble only one kernel: pack + encode in one pass (reft_parity_encode_pack)
             into a packed device copy of the shard and the parity; beside the burst two large
             DMA copies (packed shard, parity).  Needs L more bytes of device memory and no cut.

    t_ss = size / B_io (EstimateSnapshotTime) with B_io measured here; the bubble length is an
    input (the printed EstimateBubbleTime formula is not used)."""
    torch, reft, args = b.torch, b.reft, b.args
    plan, pplan, L, k = b.plan, b.pplan, b.L, b.k
    s_snap, s_copy, s_xor = b.s_pack, b.s_save, b.s_load
    n = 8192
    A = torch.randn(n, n, device=b.dev, dtype=torch.bfloat16)
    B = torch.randn(n, n, device=b.dev, dtype=torch.bfloat16)
    C = torch.empty(n, n, device=b.dev, dtype=torch.bfloat16)
    s_gemm = torch.cuda.current_stream()
    nb = reft.reft_plan_num_buckets(plan)
    t_bubble = args.bubble_ms * 1e-3

    # B_io: the direct transport's rate on this machine
    reft.reft_snapshot_pack(plan, b.p_own, None, b.host_snap, s_snap, None)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    reft.reft_snapshot_pack(plan, b.p_own, None, b.host_snap, s_snap, None)
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
        reft.reft_parity_encode(plan, b.p_all, k, b.parity, s_xor)
        reft.reft_snapshot_pack(plan, b.p_own, b.stag_save, b.host_snap, s_snap, s_copy)
        s_snap.wait_stream(s_xor)
        reft.reft_snapshot_pack(pplan, b.p_par, b.stag_psave, b.host_par, s_snap, s_copy)

    packed = torch.empty(L, dtype=torch.uint8, device=b.dev)
    p_packed = reft.ptr_array([packed])

    def iteration(policy):
        t_start = time.perf_counter()
        if policy == "fused":
            reft.reft_parity_encode_pack(plan, b.p_all, k, b.own, b.parity, packed, s_xor)
        if policy == "has":                      # layer 1: the bubble
            reft.reft_parity_encode(plan, b.p_all, k, b.parity, s_xor)
            reft.reft_snapshot_pack_range(plan, b.p_own, None, b.host_snap, 0, b_cut, s_snap, None)
        while time.perf_counter() - t_start < t_bubble:
            time.sleep(0.0005)
        done = burst()
        if policy == "naive":
            save_all_beside_compute()
        elif policy == "has":                    # layer 2: beside compute, copies only
            reft.reft_snapshot_pack_range(plan, b.p_own, b.stag_save, b.host_snap, b_cut, nb, s_snap, s_copy)
            s_snap.wait_stream(s_xor)
            reft.reft_snapshot_pack(pplan, b.p_par, b.stag_psave, b.host_par, s_snap, s_copy)
        elif policy == "fused":                  # beside compute: two large copies
            s_snap.wait_stream(s_xor)
            reft.reft_snapshot_pack(pplan, p_packed, b.stag_psave, b.host_snap, s_snap, s_copy)
            reft.reft_snapshot_pack(pplan, b.p_par, b.stag_psave, b.host_par, s_snap, s_copy)
        done.synchronize()
        t_compute_done = time.perf_counter()
        torch.cuda.synchronize()                 # the snapshot must have landed before the next one
        return t_compute_done - t_start, time.perf_counter() - t_start

    out = {}
    for policy in ("none", "naive", "has", "fused", "none", "naive", "has", "fused"):
        iteration(policy)                        # warm-up
        its = [iteration(policy) for _ in range(iterations)]
        med = sorted(x[0] for x in its)[len(its) // 2]
        full = sorted(x[1] for x in its)[len(its) // 2]
        out.setdefault(policy, []).append((med, full))
    res = {p: (min(v[0][0], v[1][0]), min(v[0][1], v[1][1])) for p, v in out.items()}
    base = res["none"][0]
    # the fused policy's host copies are what the ordinary snapshot gives (device-side comparison)
    want = torch.cat([t.reshape(-1).view(torch.uint8) for t in b.shards[b.own]])
    fused_ok = bool(torch.equal(b.host_snap.to(b.dev), want)) and bool(torch.equal(b.host_par.to(b.dev), b.parity))
    del want, packed
    return {
        "metric": "iteration time of a synthetic pipeline stage with one snapshot per iteration",
        "workload": f"config {b.wl.cfg}",
        "bubble_ms": args.bubble_ms, "burst_gemms": args.burst_gemms,
        "B_io_GBps": round(b_io / 1e9, 2), "t_ss_ms": round(t_ss * 1e3, 1),
        "cut_bytes": cut, "cut_bucket": b_cut, "buckets": nb,
        "iteration_ms": {p: round(v[0] * 1e3, 2) for p, v in res.items()},
        "iteration_plus_snapshot_tail_ms": {p: round(v[1] * 1e3, 2) for p, v in res.items()},
        "overhead_pct": {p: round(100.0 * (v[0] - base) / base, 2) for p, v in res.items()},
        "fused_snapshot_verified": fused_ok,
    }


def measured_traffic(cfg: int):
    """(HBM bytes per launch of the encode kernel, the tracked file they come from): FETCH_SIZE and
    WRITE_SIZE of a committed rocprofv3 counter run, each scaled by a copy of known size.  A
    calibrated figure from an earlier run of the same command, not measured by this run.
    (None, None) if no such profile exists for this configuration."""
    name = f"config{cfg}_kernels_hbm_traffic.txt"
    try:
        kv = {}
        for line in open(os.path.join(ROOT, "profiles", name)):
            if "=" in line and line.split("=")[0].strip().startswith("traffic_"):
                key, _, val = line.partition("=")
                kv[key.strip()] = val.strip()
        if int(kv.get("traffic_config", -1)) == cfg:
            return int(kv["traffic_bytes"]), f"profiles/{name} (rocprofv3 --pmc run of this command)"
    except (OSError, ValueError, KeyError):
        pass
    return None, None


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
        t_pack = time.perf_counter()
        others = [oracle.pack(cpu[s]) for s in range(k) if s != own]   # peers' packed shards
        all_streams = others[:own] + streams + others[own:]
        t1 = time.perf_counter()
        par = oracle.encode(all_streams)
        t_enc = time.perf_counter()
        back = oracle.unpack(streams[0], sizes)
        t_unp = time.perf_counter()
        rec = oracle.reconstruct([all_streams[s] for s in range(k) if s != lost], par)
        t_rec = time.perf_counter()
        back_lost = oracle.unpack(rec, sizes)
        t_end = time.perf_counter()
        ok = all(np.array_equal(a, b) for a, b in zip(back_lost, cpu[lost])) and \
            all(np.array_equal(a, b) for a, b in zip(back, cpu[own]))
        # per operation, with the byte accounting of the GPU stages (HBM-side bytes)
        ops = {"pack_GBps": 2 * Ls / (t_pack - t0), "encode_GBps": (k + 1) * Ls / (t_enc - t1),
               "unpack_GBps": 2 * Ls / (t_unp - t_enc), "reconstruct_GBps": (k + 1) * Ls / (t_rec - t_unp)}
        return t_end - t0, ok, {n: round(v / 1e9, 2) for n, v in ops.items()}

    out = {}
    threads_all = oracle.max_threads()
    for threads in (1, threads_all):
        oracle.set_threads(threads)
        out[threads] = one_pass()
    oracle.set_threads(1)
    t_all, ok_all, ops_all = out[threads_all]
    t_one, ok_one, ops_one = out[1]
    return {
        "value": round(4 * Ls / t_all / 1e9, 3),
        "unit": "GB/s",
        "cores": threads_all,
        "kind": "oracle",
        "sample": f"first {nsp} spans of each of the {k} shards ({Ls} bytes per shard); one pass = "
                  f"pack own + pack peers + encode + unpack + reconstruct + unpack, {t_all:.2f} s",
        "per_operation": ops_all,
        "single_thread_value": round(4 * Ls / t_one / 1e9, 3),
        "single_thread_seconds": round(t_one, 2),
        "single_thread_per_operation": ops_one,
        "verified": bool(ok_all and ok_one),
    }


if __name__ == "__main__":
    # (no sys.exit on success: with rocprofv3's memory-copy trace attached, leaving through
    # SystemExit ends in a crash inside the tool's own finalization)
    status = main()
    if status:
        sys.exit(status)
