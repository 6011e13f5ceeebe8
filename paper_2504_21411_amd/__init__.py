"""MI355X-native batched strategy-search DP (hot path of the Galvatron search engine).

`binding` wraps the C ABI of libgsearch.so, `workloads` generates the seeded synthetic
inputs, `runner` strings the entry points together for tests and benchmarks.
"""
from . import workloads  # noqa: F401  (numpy only; safe without a GPU)

__all__ = ["workloads", "binding", "runner", "build"]
