"""CPU fp64 oracle (test infrastructure).  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; the product package never does."""
