"""MI355X-native forward pass of a multi-model MoE layer over a consolidated expert pool.

``paper_2505_06481_amd.mmoe`` is the Python binding of the C-ABI library (loaded on
first use; it raises if the HIP library has not been built -- there is no CPU fallback).
``paper_2505_06481_amd.synth`` generates the seeded synthetic workloads.
"""
__all__ = ["mmoe", "synth"]
