"""MI355X-native fused linear + erf-GELU + LayerNorm (hand-written HIP, C ABI)."""
__version__ = "0.1.0"
