"""Seeded synthetic inputs shaped like the paper's rollout batches: used by the tests, the smoke
check and the benchmark.  Not part of the library; holds none of the method's arithmetic."""
