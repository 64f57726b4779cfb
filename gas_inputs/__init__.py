"""Seeded synthetic inputs shared by the tests, the benchmark and the oracle
checks: graphs, batches, index structures, features, weights, histories.
Input generation only; none of the method's arithmetic is in this package."""
from . import rng, graphs, batches, configs  # noqa: F401
