"""CPU oracle of the SMoE decode step.  Test infrastructure only: imported by
tests, the smoke check and the benchmark's cpu_baseline leg, never by the
HIP library or its Python binding."""
