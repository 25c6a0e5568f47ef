"""fp64 CPU oracle for the linear-attention hot path.  Test infrastructure only:
imported by tests/, the smoke check and the benchmark's cpu_baseline leg."""
