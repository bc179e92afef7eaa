"""MI355X-native ADC scan over product-quantized codes (Quicker ADC, arXiv 1812.09162).

``binding`` holds the ctypes front end of libqadc.so (the HIP kernels behind the C ABI
declared in ``include/qadc.h``); ``build`` compiles the library in-tree.  Nothing is imported
eagerly.
"""
__all__ = ["binding", "build"]
