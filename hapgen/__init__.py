"""Seeded synthetic inputs for the HAP per-device hot path.

This package holds only input generation (a counter-based normal generator,
the bf16 value grid the inputs live on, and the five workload shape tables).
It contains none of the method's arithmetic: no ratios, no rounding of shard
sizes, no GEMMs.  Both the CPU oracle's tests and the GPU tests draw their
inputs from here so that the two sides see identical arrays.
"""
from .rng import normal, normal_bf16, to_bf16_bits, from_bf16_bits, TensorId
from .workloads import WORKLOADS, Workload

__all__ = ["normal", "normal_bf16", "to_bf16_bits", "from_bf16_bits", "TensorId",
           "WORKLOADS", "Workload"]
