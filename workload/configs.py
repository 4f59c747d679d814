"""The five synthetic workloads: tensor inventories, span order, buckets, lost shard, values.

A *shard* is one simulated rank's training state: for every weight tensor of its tensor-parallel
share there are four state tensors (bf16 parameter, fp32 master copy, fp32 Adam first moment, fp32
Adam second moment; 2+4+4+4 = 14 bytes per parameter, the "triple extra parameters" Adam adds in
the evaluation set-up of the paper, section 7.1).  A *span* is one such state tensor's raw bytes.
The order of the spans is kind-major (all parameters, then all masters, then m, then v) unless the
workload shuffles it.  Everything here derives from ``(config id, seed)`` alone.

Nothing in this file performs any step of the method (no packing, no parity); it only lists shapes
and draws random numbers.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

BASE_SEED = 231012670
MiB = 1 << 20

# (kind name, torch dtype, bytes per element, normal std, take absolute value)
KINDS = (
    ("param", torch.bfloat16, 2, 0.02, False),
    ("master", torch.float32, 4, 0.02, False),
    ("m", torch.float32, 4, 1e-3, False),
    ("v", torch.float32, 4, 1e-6, True),
)


def config_seed(cfg: int) -> int:
    return BASE_SEED + 1000 * int(cfg)


@dataclass(frozen=True)
class Span:
    kind: int        # index into KINDS
    tensor: int      # index into Workload.tensors (canonical order)
    name: str
    numel: int
    nbytes: int


@dataclass
class Workload:
    cfg: int
    seed: int
    k: int                                   # shards in the simulated node
    tensors: List[Tuple[str, Tuple[int, ...]]]
    spans: List[Span]                        # stream order
    bucket_nbytes: List[int]                 # consecutive bucket lengths covering the stream
    lost: int                                # seed-chosen lost shard
    description: str = ""
    L: int = field(init=False)               # stream bytes per shard

    def __post_init__(self):
        self.L = sum(s.nbytes for s in self.spans)


def span_nbytes(wl: Workload) -> List[int]:
    return [s.nbytes for s in wl.spans]


# ----------------------------------------------------------------------------------------------
# tensor inventories
# ----------------------------------------------------------------------------------------------
def _llama_share(d: int, ffn: int, layers: int, kv_width: int, tp: int, vocab: int,
                 embed: bool, lm_head: bool, final_norm: bool):
    """Weight tensors of one tensor-parallel rank of a Llama-style decoder stage.

    Column-parallel q/k/v/gate/up are split on the output dimension, row-parallel o/down on the
    input dimension, RMSNorm vectors are replicated, the embedding is vocabulary-parallel.
    q/k/v and gate/up stay unfused so the inventory has more and smaller spans.
    """
    t: List[Tuple[str, Tuple[int, ...]]] = []
    if embed:
        t.append(("embed", (vocab // tp, d)))
    for l in range(layers):
        p = f"layer{l}."
        t.append((p + "q", (d // tp, d)))
        t.append((p + "k", (kv_width // tp, d)))
        t.append((p + "v", (kv_width // tp, d)))
        t.append((p + "o", (d, d // tp)))
        t.append((p + "gate", (ffn // tp, d)))
        t.append((p + "up", (ffn // tp, d)))
        t.append((p + "down", (d, ffn // tp)))
        t.append((p + "norm_attn", (d,)))
        t.append((p + "norm_mlp", (d,)))
    if final_norm:
        t.append(("final_norm", (d,)))
    if lm_head:
        t.append(("lm_head", (vocab // tp, d)))
    return t


def _tiny_partition(seed: int, total: int, parts: int = 64, n_odd: int = 8):
    """Seed-drawn cut of ``total`` elements into ``parts`` 1-D tensors with log-uniform sizes.

    At least ``n_odd`` tensors get an odd element count, so that 2-byte-element spans start at
    stream offsets that are not multiples of 4 or 16.
    """
    rng = np.random.default_rng(seed)
    raw = np.exp(rng.uniform(math.log(64.0), math.log(65536.0), parts - 1))
    raw *= (total * (parts - 1) / parts) / raw.sum()
    sizes = np.maximum(1, raw.astype(np.int64))
    odd_idx = rng.choice(parts - 1, size=n_odd, replace=False)
    sizes[odd_idx] |= 1
    last = total - int(sizes.sum())
    assert last > 0
    sizes = list(map(int, sizes)) + [last]
    return [(f"t{i}", (n,)) for i, n in enumerate(sizes)]


def _div(x: int, shrink: int, mult: int) -> int:
    """x / shrink, rounded down to a positive multiple of ``mult``."""
    return max(mult, (x // shrink) // mult * mult)


# ----------------------------------------------------------------------------------------------
# the five configurations
# ----------------------------------------------------------------------------------------------
def make_workload(cfg: int, seed: Optional[int] = None, shrink: int = 1,
                  layers: Optional[int] = None, bucket_bytes: Optional[int] = None) -> Workload:
    """Build the description of configuration ``cfg`` (0..4).

    ``shrink`` > 1 divides every model dimension (and, quadratically, the bucket sizes) so that
    the same structure can be exercised at CPU-test sizes; ``layers`` overrides the layer count.
    ``shrink == 1`` with no overrides gives the full-size configuration.
    """
    seed = config_seed(cfg) if seed is None else int(seed)
    tp = 8
    s2 = shrink * shrink

    def dims(d, ffn, kv, vocab):
        return (_div(d, shrink, tp), _div(ffn, shrink, tp), _div(kv, shrink, tp),
                _div(vocab, shrink, tp))

    shuffle = False
    random_buckets = False
    if cfg == 0:
        k = 4
        total = max(4096, 1048576 // s2)
        tensors = _tiny_partition(seed, total)
        bucket = 4 * MiB // s2
        desc = "tiny: 4 shards x 1,048,576 params, 4 MiB buckets"
    elif cfg == 1:
        k = 8
        d, ffn, kv, vocab = dims(4096, 11008, 4096, 32000)
        tensors = _llama_share(d, ffn, 32 if layers is None else layers, kv, tp, vocab,
                               embed=True, lm_head=True, final_norm=True)
        bucket = 64 * MiB // s2
        desc = "Llama-2-7B-shaped TP=8 rank share, 8 shards, 64 MiB buckets"
    elif cfg == 2:
        k = 8
        d, ffn, kv, vocab = dims(5120, 13824, 5120, 32000)
        tensors = _llama_share(d, ffn, 20 if layers is None else layers, kv, tp, vocab,
                               embed=True, lm_head=False, final_norm=False)
        bucket = 16 * MiB // s2
        shuffle = True
        desc = "Llama-2-13B-shaped TP=8 PP=2 stage 0, span order shuffled, 16 MiB buckets"
    elif cfg == 3:
        k = 8
        d, ffn, kv, vocab = dims(8192, 22016, 1024, 32000)
        tensors = _llama_share(d, ffn, 12 if layers is None else layers, kv, tp, vocab,
                               embed=True, lm_head=False, final_norm=False)
        bucket = 64 * MiB // s2
        desc = "Llama-2-34B-shaped TP=8 PP=4 stage 0 (GQA, 8 KV heads), 64 MiB buckets"
    elif cfg == 4:
        k = 8
        d, ffn, kv, vocab = dims(8192, 28672, 1024, 32000)
        tensors = _llama_share(d, ffn, 10 if layers is None else layers, kv, tp, vocab,
                               embed=True, lm_head=False, final_norm=False)
        bucket = 0
        random_buckets = True
        desc = "Llama-2-70B-shaped TP=8 PP=8 stage 0, random odd bucket lengths 1-128 MiB"
    else:
        raise ValueError(f"unknown config {cfg}")

    spans: List[Span] = []
    for kind, (_, _, esz, _, _) in enumerate(KINDS):
        for ti, (name, shape) in enumerate(tensors):
            n = int(np.prod(shape))
            spans.append(Span(kind, ti, f"{KINDS[kind][0]}:{name}", n, n * esz))

    rng = np.random.default_rng(seed)
    if shuffle:
        order = rng.permutation(len(spans))
        spans = [spans[i] for i in order]

    L = sum(s.nbytes for s in spans)
    if bucket_bytes is not None:
        bucket = int(bucket_bytes)
        random_buckets = False
    if random_buckets:
        lo = max(1, (1 << 19) // s2)
        hi = max(lo + 1, (1 << 26) // s2)
        buckets: List[int] = []
        covered = 0
        while covered < L:
            ln = 2 * int(rng.integers(lo, hi)) + 1          # odd, never a multiple of 16
            ln = min(ln, L - covered)
            buckets.append(ln)
            covered += ln
    else:
        bucket = max(1, bucket)
        nb = (L + bucket - 1) // bucket
        buckets = [bucket] * nb
        if nb:
            buckets[-1] = L - bucket * (nb - 1)

    lost = int(rng.integers(k))
    return Workload(cfg=cfg, seed=seed, k=k, tensors=tensors, spans=spans,
                    bucket_nbytes=buckets, lost=lost, description=desc)


# ----------------------------------------------------------------------------------------------
# values
# ----------------------------------------------------------------------------------------------
def fill_shard(wl: Workload, shard: int, device="cpu") -> List[torch.Tensor]:
    """Allocate and fill the state tensors of shard ``shard``; returned in span (stream) order.

    Values are drawn tensor by tensor in canonical inventory order (so shuffling the span order
    does not change them): master ~ N(0, 0.02) fp32, parameter = master rounded to bf16,
    m ~ N(0, 1e-3), v = |N(0, 1e-6)|.  Every tensor is a separate allocation.
    """
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(wl.seed + shard)
    by_key = {}
    for ti, (_, shape) in enumerate(wl.tensors):
        master = torch.empty(shape, dtype=torch.float32, device=device).normal_(0.0, 0.02, generator=gen)
        by_key[(1, ti)] = master
        by_key[(0, ti)] = master.to(torch.bfloat16)
        by_key[(2, ti)] = torch.empty(shape, dtype=torch.float32, device=device).normal_(0.0, 1e-3, generator=gen)
        by_key[(3, ti)] = torch.empty(shape, dtype=torch.float32, device=device).normal_(0.0, 1e-6, generator=gen).abs_()
    return [by_key[(s.kind, s.tensor)] for s in wl.spans]
