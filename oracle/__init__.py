"""fp64 CPU oracle for MoDA attention.  Test infrastructure only: imported by
tests/, the smoke check and the benchmark's cpu_baseline leg, never by the
product package."""
