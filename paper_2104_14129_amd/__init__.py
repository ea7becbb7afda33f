"""libactq for MI355X: per-group stochastic activation quantization (ActNN, Sec. 4-5).

``binding`` is the thin ctypes layer over the C ABI in ``include/actq.h`` (the HIP
library is loaded on first use and a missing library is an error, never a silent
CPU fallback); ``synth`` makes the seeded synthetic workloads.
"""
__all__ = ["binding", "synth", "build"]
