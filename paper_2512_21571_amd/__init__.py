"""MI355X-native Qwen3-style decoder forward pass (C-ABI library + thin binding).

Importing this package loads nothing; `paper_2512_21571_amd.binding` loads the
gfx950 shared library and fails loudly if it is missing or cannot be built.
"""
__all__ = ["binding"]
