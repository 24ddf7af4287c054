"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path's tests/bench.

This package holds shapes and random-number recipes only; none of the method's arithmetic
(no forward pass, no features, no acceptance) lives here.
"""
from .synth import *  # noqa: F401,F403
