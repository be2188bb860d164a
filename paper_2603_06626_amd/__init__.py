"""MI355X-native fixed-routing MoE expert layer (plan, permute, grouped SwiGLU FFN, combine; fwd + bwd)."""
