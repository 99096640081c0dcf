"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke run.

This package holds no arithmetic of the grouped GEMM itself: it only draws
group sizes, draws real-valued matrices and quantises them to e4m3 bytes plus
float32 block scales.  Both the CPU oracle and the HIP library consume the
bytes and scales it produces.
"""
from .configs import CONFIGS, WorkloadConfig, group_sizes, paper_group_sizes  # noqa: F401
from .quantize import make_problem, quantize_a, quantize_b  # noqa: F401
