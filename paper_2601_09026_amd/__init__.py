"""MI355X-native MGRIT (layer-parallel) hot path for neural-ODE transformers.

`workloads` draws the seeded synthetic inputs; `binding` is the thin ctypes
layer over the C-ABI HIP library (loaded lazily, on first use).
"""
__all__ = ["workloads", "binding"]
