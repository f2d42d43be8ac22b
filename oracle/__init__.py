"""CPU oracle of the sensitivity pass.  Test infrastructure only: imported by
tests/, the smoke check and the benchmark's cpu_baseline leg."""
