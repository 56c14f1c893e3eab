"""MI355X-native batched energy-cost-model evaluation (arXiv 2411.18873 hot path).

`paper_2411_18873_amd.eck` is the thin ctypes binding over the C ABI of
libeck.so (include/eck.h); `paper_2411_18873_amd.synth` generates the seeded
synthetic inputs.  Nothing is loaded at import time.
"""
__all__ = ["eck", "synth", "build"]
