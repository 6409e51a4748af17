"""Slow, exact CPU oracle for the bootstrapped-gate path.  TEST INFRASTRUCTURE ONLY:
imported by tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg, never by
the product package."""
from . import tfhe, circuits  # noqa: F401
