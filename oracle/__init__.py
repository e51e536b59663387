"""CPU oracle (test infrastructure).  Only tests, the smoke entry and the
benchmark's CPU-baseline leg may import this package; the product never does."""
