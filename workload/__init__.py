"""Seeded synthetic rank-state generator shared by the tests, the bench and the smoke run.

This package only *describes and fills* inputs: tensor inventories of a Llama-shaped rank share,
span order, bucket lengths, the lost-shard index and the random values.  It contains none of the
checkpointing method's arithmetic (no concatenation, no XOR, no slicing of streams), so both the
CPU oracle's tests and the HIP path's tests can draw inputs from it without sharing any code of the
method itself.
"""
from .configs import (  # noqa: F401
    BASE_SEED,
    KINDS,
    Span,
    Workload,
    config_seed,
    make_workload,
    fill_shard,
    span_nbytes,
)
