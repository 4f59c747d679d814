"""The pipelined step order of bench.py, checked on the CPU: the schedule is run against recording
stand-ins for streams, events and the library, and every pair of operations that touch the same
buffer must be ordered by stream order and event waits alone, in the sense the step needs (step n's
restore reads what step n's snapshot wrote, and so on)."""
import argparse
import itertools

import pytest

import bench


class FakeEvent:
    def __init__(self, enable_timing=False):
        self.at = None                      # (stream, number of operations queued on it so far)

    def record(self, stream):
        self.at = (stream, len(stream.ops))

    def synchronize(self):
        pass

    def query(self):
        return True


class FakeStream:
    def __init__(self, name):
        self.name, self.ops, self.pending = name, [], []

    def wait_event(self, ev):
        if ev.at is not None:
            self.pending.append(ev.at)      # applies to the next operation queued here

    def wait_stream(self, other):
        self.pending.append((other, len(other.ops)))


class Op:
    def __init__(self, kind, n, stream):
        self.kind, self.n, self.stream, self.before = kind, n, stream, []
        if stream.ops:
            self.before.append(stream.ops[-1])                  # stream order
        for other, count in stream.pending:                     # event waits
            if count:
                self.before.append(other.ops[count - 1])
        stream.pending = []
        stream.ops.append(self)

    def __repr__(self):
        return f"{self.kind}({self.n})"


class FakeLib:
    """Records the six operations of a step; the n-th call of a kind belongs to step n, except the
    decodes and parity restores, which the pipelined order issues late but still in step order."""

    def __init__(self):
        self.count = {}
        self.all = []

    def _op(self, kind, stream):
        n = self.count.get(kind, 0)
        self.count[kind] = n + 1
        self.all.append(Op(kind, n, stream))

    def reft_parity_encode(self, plan, ptrs, k, parity, stream):
        self._op("encode", stream)

    def reft_reconstruct_spans(self, plan, ptrs, k, lost, parity, out, stream):
        self._op("decode", stream)

    def reft_snapshot_pack(self, plan, ptrs, staging, host, pack_stream, copy_stream):
        self._op("snapshot_shard" if plan == "plan" else "snapshot_parity", copy_stream)

    def reft_restore(self, plan, host, staging, ptrs, copy_stream, unpack_stream):
        self._op("restore_shard" if plan == "plan" else "restore_parity", unpack_stream)


class FakeTorch:
    class cuda:
        Event = FakeEvent


def happens_before(a, b, seen=None):
    seen = set() if seen is None else seen
    for p in b.before:
        if p is a:
            return True
        if id(p) not in seen:
            seen.add(id(p))
            if happens_before(a, p, seen):
                return True
    return False


def run_schedule(serial, steps):
    b = object.__new__(bench.Bench)
    b.args = argparse.Namespace(serial=serial, queue_depth=1, trace_phases=False, pace_on="first")
    b.torch, b.reft = FakeTorch, FakeLib()
    b.s_save, b.s_load = FakeStream("save"), FakeStream("load")
    b.s_pack = b.s_save
    b.plan, b.pplan = "plan", "pplan"
    for name in ("p_all", "p_own", "p_par", "p_par2", "p_surv", "p_fresh_own", "p_fresh_lost", "parity",
                 "parity2", "host_snap", "host_par", "stag_save", "stag_psave", "stag_load", "stag_pload"):
        setattr(b, name, name)
    b.k, b.lost = 8, 3
    b.enc_events, b.dec_events, b.phases, b.tracing, b.step_marks = [], [], [], False, []
    b.reset_pipeline()
    for _ in range(steps):
        b.step(timed=False)
    b.drain()
    return b.reft


# buffer -> (operation that writes it, operation that reads it), both of the same step
PAIRS = {"parity": ("encode", "snapshot_parity"), "host_snap": ("snapshot_shard", "restore_shard"),
         "host_par": ("snapshot_parity", "restore_parity"), "parity2": ("restore_parity", "decode")}


@pytest.mark.parametrize("serial", [False, True])
@pytest.mark.parametrize("steps", [1, 2, 3, 7])
def test_every_buffer_is_written_then_read_then_rewritten(serial, steps):
    lib = run_schedule(serial, steps)
    by = {(o.kind, o.n): o for o in lib.all}
    for kind in ("encode", "decode", "snapshot_shard", "snapshot_parity", "restore_shard", "restore_parity"):
        assert lib.count[kind] == steps, (kind, lib.count)       # exactly one of each per step
    for buf, (writer, reader) in PAIRS.items():
        for n in range(steps):
            w, r = by[(writer, n)], by[(reader, n)]
            assert happens_before(w, r), f"{buf}: {r} may read before {w} has written"
            if n + 1 < steps:
                w2 = by[(writer, n + 1)]
                assert happens_before(r, w2), f"{buf}: {w2} may overwrite what {r} still reads"


def test_the_pipelined_order_overlaps_the_two_directions():
    """What the order is for: the parity's restore of step n is not ordered against the shard's
    snapshot of step n+1 (they share the link), nor the shard's restore against the parity's
    snapshot of its own step; and no copy is unordered against an XOR kernel (the window)."""
    lib = run_schedule(False, 6)
    by = {(o.kind, o.n): o for o in lib.all}

    def unordered(a, b):
        return not happens_before(a, b) and not happens_before(b, a)
    for n in range(1, 5):
        assert unordered(by[("restore_parity", n)], by[("snapshot_shard", n + 1)])
        assert unordered(by[("restore_shard", n)], by[("snapshot_parity", n)])
    copies = [o for o in lib.all if o.kind.startswith(("snapshot", "restore"))]
    kernels = [o for o in lib.all if o.kind in ("encode", "decode")]
    for c, x in itertools.product(copies, kernels):
        assert not unordered(c, x), f"{c} may run beside {x}"
