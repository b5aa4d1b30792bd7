"""CPU oracle (TEST INFRASTRUCTURE ONLY): only tests/, the smoke check and the benchmark's
cpu-baseline leg may import anything from this package; the product path never does."""
