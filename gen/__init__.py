"""Seeded synthetic inputs for the QuoKA chunk-attention path.

This package only *draws data*: random tensors with the shapes and geometry of
the workloads, rounded to the storage dtype.  It holds none of the method's
arithmetic (no query ranking, no key scoring, no attention) and is the one
module both the CPU oracle's tests and the HIP path's tests/bench may share.
"""
from .workloads import (  # noqa: F401
    Workload,
    bf16_round,
    bf16_bits,
    make_workload,
    make_custom,
    CONFIG_NAMES,
)


def to_torch(*a, **k):  # lazy: importing gen must not require torch
    from .device import to_torch as f
    return f(*a, **k)


def from_torch(*a, **k):
    from .device import from_torch as f
    return f(*a, **k)
