"""MI355X-native LCMA GEMM (hot path of arxiv 2605.06057)."""
