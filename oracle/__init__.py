"""CPU oracle for Superposed Decoding.  TEST INFRASTRUCTURE: only tests/, the smoke check
and the benchmark's CPU-baseline leg import this package; the product path never does."""
