"""Transfer-tuning hot path for MI355X: fused operator kernels under schedule records, and the sweep."""
