"""MI355X-native FASA decode hot path (frequency-aware sparse attention, arXiv 2602.03152).

`workload` (seeded synthetic inputs) imports without the native library; `binding`
loads the C-ABI HIP library and raises if it has not been built.
"""
__all__ = ["workload", "binding"]
