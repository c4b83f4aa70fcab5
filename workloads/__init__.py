"""Seeded synthetic attention inputs shared by the CPU oracle tests and the GPU harness.

This package only draws random tensors.  It contains none of the attention method's arithmetic and
imports neither the oracle nor the HIP binding.
"""
from .generators import (  # noqa: F401
    Workload,
    WORKLOADS,
    workload,
    gen_q_head,
    gen_kv_head,
    gen_full,
    gen_uniform_benchmark,
    gen_hybrid_benchmark,
)
