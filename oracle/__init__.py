"""CPU oracle (test infrastructure).  Not part of the product path: only tests/,
the smoke check and the benchmark's cpu_baseline leg may import this package."""
