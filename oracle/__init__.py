"""CPU oracle for the W4A16 GEMM path (test infrastructure only; see oracle_w4.c)."""
