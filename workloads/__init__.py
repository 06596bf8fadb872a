"""Seeded synthetic inputs (graphs, configurations, GEMM operands) shared by every test and by the benchmark.

Nothing in this package computes any part of the method; it only builds inputs.
"""
