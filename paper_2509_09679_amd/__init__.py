"""MI355X-native butterfly transform + low-bit quantisation (hot path of ButterflyQuant).

`binding` exposes the C ABI of libbq.so (include/bq.h) to Python; `synth` draws the seeded synthetic
workloads; `build` compiles the HIP sources in-tree.  Nothing is loaded at import time.
"""
__all__ = ["binding", "synth", "build"]
