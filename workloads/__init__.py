"""Seeded synthetic inputs shared by the tests, the CPU oracle's callers and the
benchmark.  Input generation only: no pruning-scheme validation, packing or
layer arithmetic lives in this package, and it imports neither the oracle nor
the HIP library."""
from . import configs, dtypes, masks, prng, sweeps  # noqa: F401
