"""Seeded synthetic inputs for the tests, the smoke check and the benchmark.

Not part of the product package: ``paper_1812_09162_amd`` holds only the HIP kernels, their build
script and the ctypes binding.  What is here fabricates inputs (data, codebooks, codes, inverted
lists) that both the HIP path and the CPU oracle are then given byte for byte.
"""
