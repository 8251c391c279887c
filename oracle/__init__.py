"""CPU oracle of the INT8 conv backward path.  Test infrastructure: imported only by tests/,
the smoke check and the benchmark's cpu_baseline leg."""
