"""Seeded synthetic KV-cache workloads.

This package only draws random inputs (numpy PCG64 streams) with the shapes and
value distributions of the benchmark configurations.  It contains none of the
method's arithmetic: no decomposition, no quantization, no attention.  Both the
CPU oracle's tests and the GPU harness draw their inputs from here so that the
two sides see identical bits.
"""
from .kv_synth import (  # noqa: F401
    Workload,
    WORKLOADS,
    get_workload,
    kv_pair,
    kv_tensor,
    query,
    seq_lens,
    appended_pair,
)
