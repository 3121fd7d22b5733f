"""MI355X-native ZipGEMM (fused TCA-TBE decompression + GEMM); see ``binding``."""
