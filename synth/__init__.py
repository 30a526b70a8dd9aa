"""Seeded synthetic inputs shared by the tests, the oracle checks and the benchmark.

This package holds no arithmetic of the quantizers or the GEMM: it only draws
random tensors with the shapes, value distributions and structure of the
DeepSeek-V3 layers (Section 4.2 hyper-parameters) and the MoE routing that
fixes the ragged group sizes (Section 2.1.2).
"""
