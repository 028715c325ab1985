"""CPU oracle for the ExCP compress / reconstruct hot path.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain reference that the
HIP library is checked against.  Nothing in the product package imports it and
it imports nothing from the product package; only tests, the smoke check and
the benchmark's CPU-baseline leg may call it.
"""
from .excp_oracle import *  # noqa: F401,F403
