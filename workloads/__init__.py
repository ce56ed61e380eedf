"""Seeded synthetic inputs shared by the tests, the bench and the CPU oracle.

This package is declarative only: it describes fusion patterns as op lists
(what to compute, never how), draws the runtime shapes of each benchmark
configuration from seeded generators and fills input buffers with seeded
random values.  It contains none of the arithmetic of either the HIP path or
the CPU oracle, and imports neither.
"""
from .pattern import Op, Pattern, PatternBuilder, DTYPES, OPCODES  # noqa: F401
