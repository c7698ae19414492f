"""W4A8-FP GEMM (INT4 weights x E4M3 activations) for AMD MI355X (gfx950).

``binding`` wraps the C ABI of ``include/fireq.h``; ``workloads`` draws the synthetic inputs;
``build`` compiles the HIP sources in-tree.
"""
