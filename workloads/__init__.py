"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This package holds no arithmetic of the pruning method itself (no centring, no
thresholding, no GEMV): only random draws, storage-dtype casts and layer shapes.
"""
from .synth import *  # noqa: F401,F403
