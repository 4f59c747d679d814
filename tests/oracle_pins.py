"""Pins for the CPU oracle: checks that do not come from the oracle itself.

Each ``pin_*`` function takes an oracle object (``oracle.Oracle``) and raises AssertionError when
the oracle disagrees with what the paper and the mathematics fix: hand-worked fixtures under
``tests/golden/``, closed forms, invariants (zero-sum, round trip, bucket independence,
linearity), special cases that reduce to a library routine (memcpy-like copy, ``numpy.bitwise_xor``)
and brute force in pure Python on tiny inputs.  ``test_oracle_pins.py`` runs them on the real
oracle; ``test_oracle_mutants.py`` runs them on builds with a planted mistake and expects a failure.
"""
from __future__ import annotations

import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, rest = line.partition(":")
            rows.append((key.strip(), rest.split()))
    return rows


def _hex(tokens):
    return np.array([int(t, 16) for t in tokens], dtype=np.uint8)


def _rand(rng, n):
    return rng.integers(0, 256, size=int(n), dtype=np.uint8)


# ------------------------------------------------------------------------------------------------
# golden fixtures (hand-worked)
# ------------------------------------------------------------------------------------------------
def pin_golden_xor(orc):
    """Section 4.2 Eq. 1 / Eq. 2 on the hand-worked bytes."""
    for name in ("xor_parity_worked.txt", "float_bits_worked.txt"):
        rows = _read_golden(name)
        shards = [_hex(t) for k, t in rows if k == "shard"]
        parity = [_hex(t) for k, t in rows if k == "parity"][0]
        assert np.array_equal(orc.encode(shards), parity), name
        for j in range(len(shards)):
            surv = [s for i, s in enumerate(shards) if i != j]
            assert np.array_equal(orc.reconstruct(surv, parity), shards[j]), (name, j)


def pin_golden_pack(orc):
    """Flat-vector layout (Algorithm 1, SplitParameter) on the hand-written bytes."""
    rows = _read_golden("pack_worked.txt")
    spans = [_hex(t) for k, t in rows if k == "span"]
    stream = [_hex(t) for k, t in rows if k == "stream"][0]
    assert np.array_equal(orc.pack(spans), stream)
    for k, t in rows:
        if k == "buckets":
            b = [int(x) for x in t]
            assert np.array_equal(orc.pack_bucketed(spans, b), stream), b
    outs = orc.unpack(stream, [s.size for s in spans])
    for a, b in zip(outs, spans):
        assert np.array_equal(a, b)


# ------------------------------------------------------------------------------------------------
# closed forms
# ------------------------------------------------------------------------------------------------
def pin_closed_form_parity(orc):
    L = 1000
    i = np.arange(L, dtype=np.uint64)
    # one distinct bit per shard: the parity has exactly the k low bits set
    for k in (1, 2, 3, 5, 8):
        shards = [np.full(L, 1 << s, dtype=np.uint8) for s in range(k)]
        assert np.all(orc.encode(shards) == (1 << k) - 1), k
    # k copies of the ramp i mod 256: zero for even k, the ramp for odd k
    ramp = (i % 256).astype(np.uint8)
    for k in (2, 3, 4, 7, 8):
        p = orc.encode([ramp.copy() for _ in range(k)])
        assert np.array_equal(p, ramp if k % 2 else np.zeros(L, np.uint8)), k
    # shard s = (i >> s) & 1 for s < 8: parity byte = popcount(i & 0xff) mod 2
    shards = [((i >> s) & 1).astype(np.uint8) for s in range(8)]
    pop = np.array([bin(int(x) & 0xFF).count("1") & 1 for x in i], dtype=np.uint8)
    assert np.array_equal(orc.encode(shards), pop)


def pin_closed_form_pack(orc):
    """Span t filled with byte value t: stream[o] is the index of the span owning offset o."""
    rng = np.random.default_rng(7)
    sizes = [int(x) for x in rng.integers(0, 300, size=40)]
    sizes[5] = 0
    sizes[6] = 0
    spans = [np.full(n, t, dtype=np.uint8) for t, n in enumerate(sizes)]
    ends = np.cumsum(sizes)
    L = int(ends[-1])
    owner = np.searchsorted(ends, np.arange(L), side="right").astype(np.uint8)
    assert np.array_equal(orc.pack(spans), owner)
    assert np.array_equal(orc.pack_bucketed(spans, [L]), owner)
    assert np.array_equal(orc.pack_bucketed(spans, [1] * L), owner)


# ------------------------------------------------------------------------------------------------
# invariants
# ------------------------------------------------------------------------------------------------
def pin_zero_sum(orc):
    """XOR of all shards and the parity is zero (follows from Eq. 1)."""
    rng = np.random.default_rng(11)
    for k in (2, 3, 4, 8, 9):
        for L in (0, 1, 15, 16, 17, 255, 4099, 70001):
            shards = [_rand(rng, L) for _ in range(k)]
            p = orc.encode(shards)
            assert p.size == L                      # parity volume = one protected unit
            acc = np.bitwise_xor.reduce(np.stack(shards + [p]), axis=0) if L else p
            assert not acc.any(), (k, L)


def pin_round_trip_and_bucket_independence(orc):
    """unpack(pack(x)) == x for any bucket list; the host copy does not depend on the buckets."""
    rng = np.random.default_rng(13)
    sizes = [0, 1, 2, 3, 5, 16, 17, 31, 0, 64, 255, 256, 1000, 4097, 7, 0, 33]
    spans = [_rand(rng, n) for n in sizes]
    L = sum(sizes)
    ref = np.concatenate(spans)                      # library statement of "end to end"
    assert np.array_equal(orc.pack(spans), ref)
    bucket_lists = [[L], [1] * L, [16] * (L // 16) + ([L % 16] if L % 16 else []),
                    [4096] * (L // 4096) + ([L % 4096] if L % 4096 else [])]
    for _ in range(4):
        b, left = [], L
        while left:
            n = min(left, 2 * int(rng.integers(1, 400)) + 1)
            b.append(n)
            left -= n
        bucket_lists.append(b)
    for b in bucket_lists:
        host = np.full(L + 64, 0xA5, dtype=np.uint8)          # guard band after the stream
        orc.pack_bucketed(spans, b, host)
        assert np.array_equal(host[:L], ref), b[:4]
        assert np.all(host[L:] == 0xA5)                        # never writes past L
        outs = orc.unpack(host[:L].copy(), sizes)
        for a, s in zip(outs, spans):
            assert np.array_equal(a, s)


def pin_bruteforce_reconstruct(orc):
    """Every-j reconstruct against a pure-Python triple loop on tiny inputs (Eq. 2)."""
    rng = np.random.default_rng(17)
    for k in (2, 3, 4, 8):
        for L in (0, 1, 15, 16, 17, 255, 1031):
            shards = [_rand(rng, L) for _ in range(k)]
            lists = [s.tolist() for s in shards]
            # brute-force parity: bit by bit, counting ones modulo 2
            par = []
            for i in range(L):
                byte = 0
                for bit in range(8):
                    ones = 0
                    for s in range(k):
                        ones += (lists[s][i] >> bit) & 1
                    byte |= (ones & 1) << bit
                par.append(byte)
            par = np.array(par, dtype=np.uint8)
            assert np.array_equal(orc.encode(shards), par), (k, L)
            for j in range(k):
                surv = [shards[s] for s in range(k) if s != j]
                assert np.array_equal(orc.reconstruct(surv, par), shards[j]), (k, L, j)


def pin_special_cases(orc):
    rng = np.random.default_rng(19)
    a, b, c = (_rand(rng, 5003) for _ in range(3))
    # one span: pack is a plain copy
    assert np.array_equal(orc.pack([a]), a)
    assert np.array_equal(orc.pack_bucketed([a], [5003]), a)
    # k = 1: the parity of a single shard is the shard; reconstruct with no survivors is the parity
    assert np.array_equal(orc.encode([a]), a)
    assert np.array_equal(orc.reconstruct([], a), a)
    # k = 2: numpy.bitwise_xor
    assert np.array_equal(orc.encode([a, b]), np.bitwise_xor(a, b))
    assert np.array_equal(orc.reconstruct([a], np.bitwise_xor(a, b)), b)
    # two identical shards cancel; an all-zero shard changes nothing
    assert not orc.encode([a, a.copy()]).any()
    z = np.zeros_like(a)
    assert np.array_equal(orc.encode([a, z, b, c]), orc.encode([a, b, c]))
    # order of the shards does not matter
    assert np.array_equal(orc.encode([a, b, c]), orc.encode([c, a, b]))
    # reconstruct uses every survivor: k = 3
    p = np.bitwise_xor(np.bitwise_xor(a, b), c)
    assert np.array_equal(orc.reconstruct([a, c], p), b)


def pin_linearity_and_word_width(orc):
    rng = np.random.default_rng(23)
    k, L = 5, 4096
    shards = [_rand(rng, L) for _ in range(k)]
    p0 = orc.encode(shards)
    # flipping one bit of one shard flips exactly that bit of the parity
    for (s, i, bit) in ((0, 0, 0), (2, 17, 7), (4, L - 1, 3), (1, 2048, 5)):
        mod = [x.copy() for x in shards]
        mod[s][i] ^= np.uint8(1 << bit)
        diff = np.bitwise_xor(orc.encode(mod), p0)
        assert diff[i] == (1 << bit) and np.count_nonzero(diff) == 1
    # the same parity when the shards are XORed as 16-, 32- or 64-bit words
    for dt in (np.uint16, np.uint32, np.uint64):
        acc = np.zeros(L // np.dtype(dt).itemsize, dtype=dt)
        for s in shards:
            acc ^= s.view(dt)
        assert np.array_equal(acc.view(np.uint8), p0), dt


def pin_float_payloads(orc):
    """NaN payloads, infinities, signed zeros and denormals go through as bits."""
    pats = np.array([0x7FC00123, 0xFFC0FFEE, 0x7F800000, 0xFF800000, 0x80000000, 0x00000001,
                     0x807FFFFF, 0x7F800001], dtype=np.uint32)
    a = pats.view(np.uint8).copy()
    b = np.roll(pats, 3).view(np.uint8).copy()
    c = np.roll(pats, 5).view(np.uint8).copy()
    p = orc.encode([a, b, c])
    assert np.array_equal(p.view(np.uint32), pats ^ np.roll(pats, 3) ^ np.roll(pats, 5))
    assert np.array_equal(orc.reconstruct([a, c], p).view(np.uint32), np.roll(pats, 3))
    h = np.array([0x7FC1, 0xFF80, 0x8000, 0x0001], dtype=np.uint16).view(np.uint8).copy()
    s = orc.pack([a, h, b])
    assert np.array_equal(s[a.size:a.size + h.size].view(np.uint16),
                          np.array([0x7FC1, 0xFF80, 0x8000, 0x0001], dtype=np.uint16))


def pin_padded(orc):
    """Unequal lengths: identical to the equal-length code on explicitly zero-extended shards."""
    rng = np.random.default_rng(29)
    lens = [100, 37, 0, 250, 249]
    shards = [_rand(rng, n) for n in lens]
    Lmax = max(lens)
    ext = [np.concatenate([s, np.zeros(Lmax - s.size, np.uint8)]) for s in shards]
    want = np.bitwise_xor.reduce(np.stack(ext), axis=0)
    assert np.array_equal(orc.encode_padded(shards), want)
    # beyond every other shard's end the parity is the longest shard itself
    assert np.array_equal(want[249:], shards[3][249:])


def pin_rejects(orc):
    a = np.arange(10, dtype=np.uint8)
    for bad in ([0, 10], [4, 5], [4, 7], []):
        try:
            orc.pack_bucketed([a], bad)
        except ValueError:
            continue
        raise AssertionError(f"bucket list {bad} accepted")
    try:
        orc.unpack(a, [3, 3])
    except ValueError:
        pass
    else:
        raise AssertionError("unpack accepted sizes that do not sum to the stream length")


# ------------------------------------------------------------------------------------------------
# rotated placement of the parity (section 4.2)
# ------------------------------------------------------------------------------------------------
def _segments(shard, k):
    """The k-1 zero-extended segments of a shard, by numpy slicing."""
    L = shard.size
    Lseg = -(-L // (k - 1))
    padded = np.concatenate([shard, np.zeros((k - 1) * Lseg - L, np.uint8)])
    return padded.reshape(k - 1, Lseg) if Lseg else np.zeros((k - 1, 0), np.uint8)


def pin_golden_rotated(orc):
    """Eq. 1 for the first member and the hand-worked units of the others."""
    rows = _read_golden("rotated_parity_worked.txt")
    shards = [_hex(t) for k, t in rows if k == "shard"]
    parities = [_hex(t) for k, t in rows if k == "parity"]
    k, L = len(shards), shards[0].size
    for i in range(k):
        assert np.array_equal(orc.encode_rotated(shards, i), parities[i]), i
    for lost in range(k):
        sh = [None if j == lost else shards[j] for j in range(k)]
        pa = [None if j == lost else parities[j] for j in range(k)]
        assert np.array_equal(orc.reconstruct_rotated(sh, pa, lost, L), shards[lost]), lost


def pin_rotated_invariants(orc):
    rng = np.random.default_rng(31)
    for k in (2, 3, 4, 5, 8):
        for L in (0, 1, 6, 7, 41, 42, 43, 1000, 4099):
            shards = [_rand(rng, L) for _ in range(k)]
            parities = [orc.encode_rotated(shards, i) for i in range(k)]
            Lseg = -(-L // (k - 1))
            # redundancy per member = shard size / (k-1), rounded up
            assert all(p.size == Lseg == orc.segment_bytes(L, k) for p in parities), (k, L)
            segs = [_segments(s, k) for s in shards]
            # Eq. 1 literally: the first member's unit is segment 0 of every other member
            want0 = np.zeros(Lseg, np.uint8)
            for j in range(1, k):
                want0 ^= segs[j][0]
            assert np.array_equal(parities[0], want0), (k, L)
            # every segment of every shard is protected exactly once: the XOR of all units equals
            # the XOR of all segments of all shards
            allp = np.zeros(Lseg, np.uint8)
            for p in parities:
                allp ^= p
            alls = np.zeros(Lseg, np.uint8)
            for sg in segs:
                for r in range(k - 1):
                    alls ^= sg[r]
            assert np.array_equal(allp, alls), (k, L)
            # a unit never covers its own member: changing shard i leaves unit i unchanged
            for i in (0, k - 1):
                mod = [s.copy() for s in shards]
                if L:
                    mod[i] ^= 0xFF
                assert np.array_equal(orc.encode_rotated(mod, i), parities[i]), (k, L, i)
            # any one member lost: decoded from the others alone (its own data poisoned)
            for lost in range(k):
                sh = [(_rand(rng, L) if j == lost else shards[j]) for j in range(k)]
                pa = [(_rand(rng, Lseg) if j == lost else parities[j]) for j in range(k)]
                assert np.array_equal(orc.reconstruct_rotated(sh, pa, lost, L), shards[lost]), \
                    (k, L, lost)
    # two members: the unit of one is the other's whole shard (erasure coding degenerates to the
    # redundant copy of ARC)
    a, b = _rand(rng, 77), _rand(rng, 77)
    assert np.array_equal(orc.encode_rotated([a, b], 0), b)
    assert np.array_equal(orc.encode_rotated([a, b], 1), a)


def pin_rotated_bruteforce(orc):
    """Pure-Python loops over every byte, with the segment map written as a table."""
    rng = np.random.default_rng(37)
    for k in (3, 4):
        # table[i][j] = segment of shard j protected on member i, built from the two rules
        # "first member takes segment 0 of all" and "each (j, r) once", filled greedily
        table = [[None] * k for _ in range(k)]
        for j in range(k):
            r = 0
            for i in range(k):
                if i != j:
                    table[i][j] = r
                    r += 1
        for L in (5, 12, 13):
            shards = [_rand(rng, L).tolist() for _ in range(k)]
            Lseg = -(-L // (k - 1))
            for i in range(k):
                unit = []
                for x in range(Lseg):
                    v = 0
                    for j in range(k):
                        if j != i:
                            y = table[i][j] * Lseg + x
                            if y < L:
                                v ^= shards[j][y]
                    unit.append(v)
                got = orc.encode_rotated([np.array(s, np.uint8) for s in shards], i)
                assert got.tolist() == unit, (k, L, i)


# ------------------------------------------------------------------------------------------------
# collaborative protection (section 4.2, last paragraph)
# ------------------------------------------------------------------------------------------------
def _holdings(orc, shards, arc_offsets, aec):
    k = len(shards)
    dups = [[shards[(i + d) % k] for i in range(k)] for d in arc_offsets]
    units = [orc.encode_rotated(shards, i) for i in range(k)] if aec else None
    return dups, units


def _survivors_only(rows, lost):
    return [None if i in lost else a for i, a in enumerate(rows)]


def pin_golden_collab(orc):
    """The hand-worked cases: which segments come back, and their bytes."""
    shards = [_hex(t) for k, t in _read_golden("rotated_parity_worked.txt") if k == "shard"]
    k, L = len(shards), shards[0].size
    rows = _read_golden("collab_recovery_worked.txt")
    cases = []
    for key, t in rows:
        if key == "case":
            offs = [] if t[0] == "-" else [int(x) for x in t[0].split(",")]
            cases.append({"offs": offs, "aec": t[1] == "1", "lost": [int(x) for x in t[2].split(",")],
                          "unknown": int(t[3]), "rec": {}})
        else:
            cases[-1]["rec"][int(t[0])] = t[1:]
    assert len(cases) == 7
    for c in cases:
        dups, units = _holdings(orc, shards, c["offs"], c["aec"])
        rec, unknown, seg = orc.collab_recover(
            _survivors_only(shards, c["lost"]), [_survivors_only(d, c["lost"]) for d in dups],
            c["offs"], None if units is None else _survivors_only(units, c["lost"]), c["lost"], L)
        assert unknown == c["unknown"], c
        assert sorted(rec) == sorted(c["lost"]) == sorted(c["rec"]), c
        for x, toks in c["rec"].items():
            for o, tok in enumerate(toks):
                known = bool(seg[x][o // 2])
                assert known == (tok != "??"), (c, x, o)
                if known:
                    assert rec[x][o] == int(tok, 16), (c, x, o)


def pin_collab_bruteforce(orc):
    """Which segments are determined by what survives, by exhaustive search: shards of k-1
    one-bit segments, every value of the lost shards tried against every surviving copy and unit
    (the units recomputed with plain Python XOR from the segment map written as a table).  A
    segment is recoverable iff all candidates that fit agree on it; the oracle must find exactly
    those, with the right values, for every set of one, two or three lost members."""
    import itertools
    rng = np.random.default_rng(53)
    for k in (3, 4, 5):
        nseg = k - 1
        table = [[None] * k for _ in range(k)]          # table[i][j]: segment of j covered on i
        for j in range(k):
            r = 0
            for i in range(k):
                if i != j:
                    table[i][j] = r
                    r += 1
        truth = [rng.integers(0, 2, size=nseg, dtype=np.uint8) for _ in range(k)]

        def unit_of(i, sh):
            v = 0
            for j in range(k):
                if j != i:
                    v ^= int(sh[j][table[i][j]])
            return v
        strategies = [([1], True), ([1], False), ([], True), ([1, 2], False), ([2], True)]
        if k >= 4:
            strategies.append(([1, 3], True))
        for offs, aec in strategies:
            offs = [d for d in offs if d < k]
            dups, units = _holdings(orc, truth, offs, aec)
            for nlost in (1, 2, 3):
                if nlost >= k:
                    continue
                for lost in itertools.combinations(range(k), nlost):
                    # exhaustive: all values of the lost shards that fit what survives
                    fits = []
                    for bits in itertools.product((0, 1), repeat=nlost * nseg):
                        cand = [t.copy() for t in truth]
                        for n, x in enumerate(lost):
                            cand[x] = np.array(bits[n * nseg:(n + 1) * nseg], dtype=np.uint8)
                        ok = True
                        for d in offs:
                            for i in range(k):
                                if i not in lost and not np.array_equal(cand[(i + d) % k], truth[(i + d) % k]):
                                    ok = False
                        if aec:
                            for i in range(k):
                                if i not in lost and unit_of(i, cand) != unit_of(i, truth):
                                    ok = False
                        if ok:
                            fits.append(cand)
                    assert fits, "the truth itself must fit"
                    rec, unknown, seg = orc.collab_recover(
                        _survivors_only(truth, lost), [_survivors_only(d, lost) for d in dups], offs,
                        None if units is None else _survivors_only(units, lost), lost, nseg)
                    n_unknown = 0
                    for x in lost:
                        for r in range(nseg):
                            determined = len({int(c[x][r]) for c in fits}) == 1
                            assert bool(seg[x][r]) == determined, (k, offs, aec, lost, x, r)
                            if determined:
                                assert rec[x][r] == truth[x][r], (k, offs, aec, lost, x, r)
                            else:
                                n_unknown += 1
                    assert unknown == n_unknown, (k, offs, aec, lost)


def pin_collab_invariants(orc):
    """Random bytes, ragged lengths: one loss is always recovered by either strategy alone; two
    redundant copies with different offsets survive any two losses (k >= 3); a shard is never
    rebuilt from its own lost holdings (they are poisoned)."""
    import itertools
    rng = np.random.default_rng(59)
    for k in (3, 4, 6):
        for L in (1, 7, 41, 1000):
            shards = [_rand(rng, L) for _ in range(k)]
            for offs, aec, max_lost in (([1], False, 1), ([], True, 1), ([1, 2], False, 2), ([2], True, 1)):
                dups, units = _holdings(orc, shards, offs, aec)
                for nlost in range(1, max_lost + 1):
                    for lost in itertools.combinations(range(k), nlost):
                        sh = [(_rand(rng, L) if i in lost else a) for i, a in enumerate(shards)]
                        du = [[(_rand(rng, L) if i in lost else a) for i, a in enumerate(d)] for d in dups]
                        un = None if units is None else \
                            [(_rand(rng, a.size) if i in lost else a) for i, a in enumerate(units)]
                        rec, unknown, seg = orc.collab_recover(sh, du, offs, un, lost, L)
                        assert unknown == 0 and seg.all(), (k, L, offs, aec, lost)
                        for x in lost:
                            assert np.array_equal(rec[x], shards[x]), (k, L, offs, aec, lost, x)


ALL_PINS = [pin_golden_xor, pin_golden_pack, pin_closed_form_parity, pin_closed_form_pack,
            pin_zero_sum, pin_round_trip_and_bucket_independence, pin_bruteforce_reconstruct,
            pin_special_cases, pin_linearity_and_word_width, pin_float_payloads, pin_padded,
            pin_rejects, pin_golden_rotated, pin_rotated_invariants, pin_rotated_bruteforce,
            pin_golden_collab, pin_collab_bruteforce, pin_collab_invariants]
