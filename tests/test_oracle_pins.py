"""The CPU oracle against its pins (no GPU).  See ``oracle_pins.py`` for what each pin fixes."""
import numpy as np
import pytest

import oracle
from oracle_pins import ALL_PINS
from workload import make_workload, fill_shard


@pytest.mark.parametrize("pin", ALL_PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin(oracle.default())


@pytest.mark.parametrize("threads", [1, 3, 8])
def test_pins_hold_with_threads(threads):
    """The optional OpenMP split of the byte range does not change any result."""
    orc = oracle.default()
    orc.set_threads(threads)
    try:
        rng = np.random.default_rng(threads)
        k, L = 4, (3 << 20) + 5                    # above the size at which the split is used
        shards = [rng.integers(0, 256, L, dtype=np.uint8) for _ in range(k)]
        p = orc.encode(shards)
        assert not np.bitwise_xor.reduce(np.stack(shards + [p]), axis=0).any()
        assert np.array_equal(orc.reconstruct(shards[1:], p), shards[0])
        assert np.array_equal(orc.pack(shards), np.concatenate(shards))
        outs = orc.unpack(np.concatenate(shards), [L] * k)
        assert all(np.array_equal(a, b) for a, b in zip(outs, shards))
    finally:
        orc.set_threads(1)


@pytest.mark.parametrize("cfg,shrink,layers", [(0, 1, None), (1, 32, 2), (2, 32, 3), (3, 32, 2),
                                               (4, 32, 2)])
def test_workload_shaped_inputs(cfg, shrink, layers):
    """Zero-sum, round trip and lost-shard reconstruct on inputs shaped like each configuration."""
    wl = make_workload(cfg, shrink=shrink, layers=layers)
    streams = []
    for s in range(wl.k):
        spans = [oracle.as_bytes(t) for t in fill_shard(wl, s)]
        assert [a.size for a in spans] == [sp.nbytes for sp in wl.spans]
        host = oracle.pack_bucketed(spans, wl.bucket_nbytes)
        assert np.array_equal(host, np.concatenate(spans))
        if s == 0:
            outs = oracle.unpack(host, [a.size for a in spans])
            assert all(np.array_equal(a, b) for a, b in zip(outs, spans))
        streams.append(host)
    assert all(st.size == wl.L for st in streams)
    p = oracle.encode(streams)
    assert not np.bitwise_xor.reduce(np.stack(streams + [p]), axis=0).any()
    j = wl.lost
    rec = oracle.reconstruct([st for s, st in enumerate(streams) if s != j], p)
    assert np.array_equal(rec, streams[j])
    # random shards do not cancel: the parity is not trivially zero
    assert np.count_nonzero(p) > 0.9 * p.size
