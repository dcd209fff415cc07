"""Seeded synthetic workloads: model shapes and input generators.

This package holds no arithmetic of the decode path itself.  It only draws
random bytes / numbers with the distributions the benchmark configurations
prescribe, so that the CPU oracle and the HIP path can be fed identical inputs
without sharing any code of their own.
"""
from .configs import CONFIGS, ModelDims, WindowConfig  # noqa: F401
from . import synth  # noqa: F401
