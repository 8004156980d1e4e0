"""Jagged Flash Attention for AMD MI355X (gfx950): thin Python binding over the C-ABI library libjfa.so.

Importing the package loads nothing; the HIP library is loaded on first use of
``paper_2409_15373_amd.binding`` and a missing library raises (there is no CPU fallback).
"""
__version__ = "0.1.0"
