"""MI355X-native fused log-domain Sinkhorn (squared-Euclidean entropic OT).

The compute lives in ``libflashsink.so`` (hand-written HIP for gfx950 behind a
C ABI, see ``include/flashsink.h``); ``paper_2602_03067_amd.binding`` is the thin
ctypes layer with the same entry-point names.  Importing this package does not
load the library; ``binding`` does, and fails loudly if it is missing.
"""
__all__ = ["binding", "workloads", "build"]
