"""CPU oracle for register-allocation verification.  TEST INFRASTRUCTURE ONLY:
only tests, the smoke check and the benchmark's CPU-baseline leg may import it."""
