"""TEST INFRASTRUCTURE -- the CPU oracle.  Not part of the product path: only
tests, the smoke check and the benchmark's cpu_baseline leg may import it."""
