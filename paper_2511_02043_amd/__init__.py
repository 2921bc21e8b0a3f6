"""MI355X-native fused attention-variant forward kernels behind a C-ABI library.

`binding` loads the built library lazily (import of this package never needs a GPU).
"""
__all__ = ["inputs", "binding"]
