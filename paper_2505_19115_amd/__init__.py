"""MI355X-native NVFP4 quantized linear layer (hot path of "FP4 All the Way")."""
