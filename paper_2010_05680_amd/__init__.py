"""MI355X-native batch-reduction kernels (masked softmax, add-bias-LayerNorm)."""
