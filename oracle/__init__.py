"""CPU oracle (test infrastructure).  Only tests, the smoke check and the bench's cpu_baseline
leg may import this package; the product path never does."""
