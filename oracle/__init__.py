"""CPU oracle of the SpeCa sampling step.  TEST INFRASTRUCTURE ONLY: imported by
tests/, by the smoke check and by the benchmark's cpu_baseline leg; never by the
product path.  Shares no code with the HIP library."""
