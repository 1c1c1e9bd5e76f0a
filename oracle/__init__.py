"""CPU oracle for the LIF-SNN training step.  TEST INFRASTRUCTURE ONLY: imported
by tests, the smoke check and the benchmark's cpu_baseline leg, never by the
product path, and independent of the HIP kernels."""
