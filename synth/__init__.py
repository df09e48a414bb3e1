"""Seeded input generators shared by the tests, the oracle's callers and the bench.

Holds none of the verification method's arithmetic.
"""
from . import philox, workloads  # noqa: F401
