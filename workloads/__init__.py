"""Seeded synthetic workloads shared by the tests and the benchmark."""
from .synth import *  # noqa: F401,F403
from .synth import WORKLOADS, Workload, Inputs, generate, f32_to_bf16_bits, small_variant
