"""CPU oracle for the fused linear cross-entropy path.  TEST INFRASTRUCTURE:
only the tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; the product path never does."""
