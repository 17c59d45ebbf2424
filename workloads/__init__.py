"""Seeded synthetic inputs (masks, Q/K/V) shared by the CPU oracle's tests and the GPU path's tests.

This package holds input generation only: no attention arithmetic, no block reduction, no index
construction.  Every generator is a pure function of its arguments and an integer seed.
"""
from .qkv import make_qkv, f32_to_bf16_bits  # noqa: F401
from . import masks  # noqa: F401
from .configs import CONFIGS, make_config, small_variant  # noqa: F401
