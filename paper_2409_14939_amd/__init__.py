"""MI355X-native block aggregation (forward / backward neighbour aggregation
over sampled mini-batch blocks).  The work is done by libfastgl_agg.so
(hand-written HIP for gfx950); `binding` is a thin ctypes layer over its C ABI.
"""
__all__ = ["binding", "build"]
