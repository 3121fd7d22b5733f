"""MI355X-native ZipGEMM: fused TCA-TBE decompression + GEMM (ZipServ, ASPLOS'26).

``binding``  ctypes wrappers with the names of the C ABI in include/zipserv.h
``inputs``   seeded synthetic weights / activations
``build``    builds libzipserv_hip.so with hipcc for gfx950
"""
