"""Seeded synthetic input generators for the polysemous-code search path.

This package holds *inputs only*: raw vectors, random bit strings and the
named workload shapes.  It contains none of the method's arithmetic (no
quantizer, no Hamming distance, no look-up table, no ranking), so both the
CPU oracle's tests and the HIP path's tests may draw their inputs from it
without sharing any of the computation under test.
"""
from .generators import (  # noqa: F401
    CONFIGS,
    WorkloadConfig,
    mixture_centres,
    sift_like,
    sift_like_torch,
    relu_like,
    random_codes,
    get_config,
)
