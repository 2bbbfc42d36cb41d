"""MI355X-native dynamic sparse attention for long-context prefill (MInference 1.0 hot path).

`binding` is the thin ctypes layer over the C-ABI library (libminf.so, built
from csrc/ by __graft_entry__.build()); `workloads` draws the seeded synthetic
inputs; `costmodel` counts the tiles a set of indices costs.
"""
__version__ = "0.1.0"
