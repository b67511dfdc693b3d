"""MixAttention KV-cache attention for MI355X (gfx950): C-ABI library + thin binding.

`workloads` (seeded synthetic inputs) imports without the compiled library; the
binding in `binding` loads `libmixattn.so` and fails loudly when it is missing.
"""

__all__ = ["workloads", "binding"]
