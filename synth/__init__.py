"""Seeded synthetic inputs (random numbers, generators, level-format packing).

Shared by the CPU oracle's tests and the GPU path's tests/bench; holds none of the
contractions' arithmetic.
"""
from . import rng, formats, generate  # noqa: F401
from .formats import LevelTensor, D, CU, CN, S, pack_coo, pack_csf3, pack_csr, pack_dcsr  # noqa: F401
