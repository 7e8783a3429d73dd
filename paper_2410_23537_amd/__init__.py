"""MI355X-native quantized, paged KV-cache decode path (quantize-and-write,
paged single-query attention, page dequantizer) behind a C-ABI library.

Importing the package does not load the HIP library; ``paper_2410_23537_amd.binding``
does, and raises if the library has not been built.
"""
