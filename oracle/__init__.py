"""CPU checker (test infrastructure).  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import this package; the product never does."""
