"""MI355X-native NVFP4 quantize-and-GEMM hot path (arXiv 2509.25149).

``binding`` wraps the C ABI of ``libnvfp4_hip.so``; ``synth`` holds the seeded
input generators; ``build`` compiles the library.  Importing the package does
not load the library; the first call does, and raises if it is missing.
"""
