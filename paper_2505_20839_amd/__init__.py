"""W4A8-FP GEMM (INT4 weights x E4M3 activations) for AMD MI355X (gfx950)."""
