"""CPU oracle of the pooled decoder step.  TEST INFRASTRUCTURE: only tests, the
smoke check and the benchmark's cpu_baseline leg may import this package."""
