"""Host logic of collaborative protection (section 4.2, last paragraph), on the CPU: the library's
recovery plan against the oracle's recovery procedure for every set of lost members, and the
staged transport's copy counts for the five configurations (no GPU: host-only plans)."""
import itertools

import numpy as np
import pytest

import oracle
import paper_2310_12670_amd as reft
from workload import make_workload, span_nbytes

STRATEGIES = [([1], True), ([1], False), ([], True), ([1, 2], False), ([2], True), ([1, 3], True),
              ([2, 3], False), ([1, 2], True)]


@pytest.mark.parametrize("k", [2, 3, 4, 5, 6])
def test_plan_agrees_with_the_oracle_for_every_loss(k):
    """A lost member has a step exactly when the oracle recovers all of its segments; a copy step
    names a surviving member that really keeps the duplicate; the verdict is REFT_EUNRECOVERABLE
    exactly when the oracle leaves a segment unknown."""
    rng = np.random.default_rng(k)
    # every one of the k-1 segments holds bytes (with a stream so short that the last segment is
    # empty, the unit that covers it is not missed and the oracle recovers more than the plan,
    # which does not look at lengths, promises)
    L = 3 * (k - 1) - 1
    shards = [rng.integers(0, 256, size=L, dtype=np.uint8) for _ in range(k)]
    for offs, aec in STRATEGIES:
        offs = [d for d in offs if d < k]
        dups = [[shards[(i + d) % k] for i in range(k)] for d in offs]
        units = [oracle.encode_rotated(shards, i) for i in range(k)] if aec else None
        for nlost in range(1, k):
            for lost in itertools.combinations(range(k), nlost):
                hide = lambda rows: [None if i in lost else a for i, a in enumerate(rows)]
                rec, unknown, seg = oracle.collab_recover(
                    hide(shards), [hide(d) for d in dups], offs, None if units is None else hide(units),
                    lost, L)
                steps, ok = reft.reft_recovery_plan(k, offs, aec, lost)
                whole = [x for x in lost if seg[x].all()]
                assert sorted(s[0] for s in steps) == whole, (k, offs, aec, lost)
                assert ok == (unknown == 0) == (len(whole) == len(lost)), (k, offs, aec, lost)
                for member, how, source, which in steps:
                    if how == reft.REFT_RECOVER_COPY:
                        assert source not in lost and (source + offs[which]) % k == member
                        assert np.array_equal(dups[which][source], shards[member])
                    else:
                        assert how == reft.REFT_RECOVER_DECODE and aec and len(lost) == 1
                    assert np.array_equal(rec[member], shards[member])


def test_two_copies_survive_any_two_losses_and_a_copy_plus_parity_does_not():
    for k in range(3, 10):
        for lost in itertools.combinations(range(k), 2):
            assert reft.reft_recovery_plan(k, [1, 2], False, lost)[1]
            adjacent = (lost[1] - lost[0]) % k == 1 or (lost[0] - lost[1]) % k == 1
            assert reft.reft_recovery_plan(k, [1], True, lost)[1] == (not adjacent), (k, lost)
    # three losses are beyond two strategies (some member loses both of its duplicates' holders)
    assert not reft.reft_recovery_plan(4, [1, 2], False, (0, 1, 2))[1]
    assert "cannot be recovered" in reft.reft_last_error()


def test_plan_rejects_bad_arguments():
    for k, offs in ((1, []), (33, []), (4, [0]), (4, [4])):
        with pytest.raises(reft.ReftError) as e:
            reft.reft_recovery_plan(k, offs, True, [0])
        assert e.value.code == reft.REFT_EINVAL


def test_staged_work_of_the_configurations():
    """One copy per tensor for the Llama-shaped configurations (no copy is split at a bucket
    boundary, no gather kernel runs); runs of small tensors are gathered."""
    reft.reft_set_tunable("host_only_plans", 1)
    try:
        for cfg in (1, 2, 3, 4):
            wl = make_workload(cfg)
            plan = reft.reft_plan_create(span_nbytes(wl), wl.bucket_nbytes)
            gathers, copies = reft.reft_plan_staged_work(plan)
            reft.reft_plan_destroy(plan)
            # (a small tensor that straddles a bucket boundary travels as two copies)
            assert gathers == 0 and len(wl.spans) <= copies <= len(wl.spans) + 2, (cfg, gathers, copies)
        # 16 full buckets of 16 tensors of 1 KiB each: every bucket is one gathered run, one copy
        plan = reft.reft_plan_create([1024] * 256, None, 16384)
        gathers, copies = reft.reft_plan_staged_work(plan)
        reft.reft_plan_destroy(plan)
        assert gathers == copies == 16
        # a large tensor cut by many buckets is one copy; the small ones around it too few to gather
        plan = reft.reft_plan_create([100, 10 << 20, 100], None, 1 << 20)
        assert reft.reft_plan_staged_work(plan) == (0, 3)
        reft.reft_plan_destroy(plan)
    finally:
        reft.reft_set_tunable("host_only_plans", 0)
