"""CPU oracle for the HLQ LUT GEMV/GEMM path: test infrastructure, not product code."""
