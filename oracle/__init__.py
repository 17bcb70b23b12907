"""CPU oracle of the BPDQ per-layer pass.  TEST INFRASTRUCTURE ONLY: imported by the
tests, the smoke check and the benchmark's cpu_baseline leg, never by the library."""
