"""MI355X-native hot path of Dynamic Mask Attention (arxiv 2508.02124).

`workloads` draws the seeded synthetic inputs; `binding` marshals arguments
into the C-ABI library built from `csrc/` (it raises if the library is absent:
there is no CPU fallback).
"""
__version__ = "0.1.0"
