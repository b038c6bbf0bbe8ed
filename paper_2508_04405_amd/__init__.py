"""MI355X-native W6A6 / W6A8 quantized linear layer (GEMM + decode GEMV)."""
