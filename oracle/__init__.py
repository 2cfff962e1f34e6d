"""CPU oracle for the prefix-cached prefill path.  Test infrastructure only:
imported by tests/, the smoke check and the benchmark's cpu_baseline leg, never
by the product path.  It imports nothing from the HIP package."""
