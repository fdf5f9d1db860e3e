"""MI355X-native bit-serial LUT GEMV/GEMM over HLQ weights (ELUTQ, arXiv 2510.19482)."""
