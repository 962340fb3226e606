"""MI355X-native block-wise causal attention for Next-Frame Diffusion (hot path only)."""
