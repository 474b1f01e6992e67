"""MI355X-native fused VQ decode attention (VecInfer hot path).

``paper_2510_06175_amd.binding`` exposes the C-ABI library's entry points under
the same names; ``paper_2510_06175_amd.synth`` draws the seeded test inputs.
Importing this package loads nothing native: the library is loaded on first use
and a missing build is an error, never a fallback.
"""
__all__ = ["binding", "synth", "build"]
