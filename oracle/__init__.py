"""CPU oracle for the IVF retrieval path.  Test infrastructure: imported only by
tests, the smoke check and the benchmark's cpu_baseline leg."""
