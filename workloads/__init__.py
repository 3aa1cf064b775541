"""Seeded synthetic inputs shaped like the paper's MoE layers (Table 1).

This package only *produces inputs* (tokens, gate assignments, rotation
matrices, an expert stand-in).  It contains none of the method's arithmetic
(no hashing, grouping, centroid or restore step) and is the one module that
the CPU oracle's tests and the HIP path's tests/bench both draw from.
"""
from .synth import CONFIGS, Workload, config, generate, expert_standin, storage_to_f32  # noqa: F401
