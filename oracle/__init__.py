"""CPU oracle (FP64 triple-loop GEMM).  Test infrastructure only: imported by tests,
the smoke check and the benchmark's cpu_baseline leg, never by the product path."""
