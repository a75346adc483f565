"""Seeded synthetic workloads shared by the tests, the benchmark and the smoke run.

This package holds the workload table and the input generators only.  It contains
none of the method's arithmetic (no Hilbert keys, no pooling, no softmax, no
selection): both the CPU oracle and the HIP path are fed from here, and neither of
them is imported by it.
"""
from .configs import CONFIGS, Workload, derived_sizes  # noqa: F401
from .synth import make_qkv, to_bf16_bits, bf16_bits_to_f32, round_to_bf16  # noqa: F401
