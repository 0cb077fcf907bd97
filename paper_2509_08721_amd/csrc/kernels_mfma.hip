// MFMA (bf16, tile-aligned) kernels.
