"""fp64 CPU oracle of the CCE- loss.  TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke
check and the benchmark's cpu_baseline leg; never by the product package."""
