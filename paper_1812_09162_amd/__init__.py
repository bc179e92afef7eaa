"""MI355X-native ADC scan over product-quantized codes (Quicker ADC, arXiv 1812.09162).

``binding`` holds the ctypes front end of libqadc.so (the HIP kernels behind the C ABI
declared in ``include/qadc.h``); ``synth`` fabricates seeded inputs; ``build`` compiles
the library in-tree.  Nothing is imported eagerly so that ``synth`` can be used
without the library.
"""
__all__ = ["binding", "synth", "build"]
