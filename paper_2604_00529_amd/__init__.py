"""MI355X-native MX quantization, Slice-and-Scale, fake-quant and dequantization."""
