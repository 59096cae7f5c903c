"""Seeded synthetic inputs for the selective-recompute path.

This package only *produces inputs* (chunk caches, prompt queries, recompute
rows).  It holds none of the five stages' arithmetic and is imported by the
tests, the benchmark and the smoke check; neither the CPU oracle nor the HIP
library imports it.
"""
from .synth import (  # noqa: F401
    PRESETS,
    Workload,
    WorkloadSpec,
    bf16_bits_to_f64,
    f64_to_bf16_bits,
    make_recompute_inputs,
    make_workload,
    preset,
    rope_at,
    to_f64,
    to_storage,
)
