"""fp64 CPU oracle of the 2BW stage hot path.  TEST INFRASTRUCTURE ONLY: only tests, the smoke
check and the benchmark's CPU-baseline leg may import it; the product path never does."""
