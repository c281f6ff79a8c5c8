"""Seeded synthetic input generators shared by the tests, the oracle-side test
helpers and the benchmark.  Holds no protocol arithmetic."""
from . import configs, masks, rng  # noqa: F401
