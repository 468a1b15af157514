"""fp64 CPU oracle for dilated flash attention.  Test infrastructure only: imported by
tests, the smoke check and the benchmark's CPU-baseline leg, never by the GPU package."""
