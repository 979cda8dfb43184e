"""Exact fused attention for AMD MI355X (gfx950): thin Python binding over the C-ABI HIP library.

`inputs` (synthetic data) imports nothing native; everything else goes through
`binding`, which loads `libfa_mi355.so` and raises if it has not been built.
"""
__all__ = ["binding", "inputs"]
