"""Fused 8-bit optimizer step for MI355X (gfx950): Python binding of the C-ABI library.

`from paper_2412_01195_amd import q8opt` loads the HIP library; importing this package or
its `synth` module alone does not.
"""
__all__ = ["q8opt", "synth"]
