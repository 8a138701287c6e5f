"""MI355X-native Topological Synapse hot path (Warp-Cortex, Sec. 3.3).

`paper_2601_01298_amd.binding` is the thin ctypes layer over the C-ABI library
built from `csrc/`; `paper_2601_01298_amd.synthetic` holds the seeded input
generators.  The library is loaded on first use, not at import.
"""
__all__ = ["binding", "synthetic"]
