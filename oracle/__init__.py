"""CPU oracle for SubNet-stream inference and the SushiSched policy — TEST INFRASTRUCTURE ONLY.

Written from the paper (arXiv 2306.17266) and the textbook definition of a CNN
forward pass.  Nothing in the GPU library imports this package and this package
imports nothing from the GPU library.  Allowed callers: tests/, the smoke check
and the CPU-baseline leg of the benchmark.
"""
