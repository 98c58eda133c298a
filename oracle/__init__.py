"""CPU oracle of the hot path.  Test infrastructure: imported only by tests,
the smoke check and the benchmark's CPU-baseline leg."""
