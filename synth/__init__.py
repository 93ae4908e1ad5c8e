"""Seeded synthetic workloads: member descriptions, parameters and images.

Shared by the CPU oracle's tests and the GPU library's tests and benchmark as
a source of inputs only; it contains none of the ensemble method's arithmetic.
"""
from . import rng, nets, weights  # noqa: F401

BASE_SEED = 220814049
