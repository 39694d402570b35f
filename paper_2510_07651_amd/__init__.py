"""MI355X-native OBCache hot path: window-attention saliency scoring, per-head top-k, K/V compaction.

The compute lives in the HIP library (csrc/, C ABI in include/obcache.h); `binding`
is a thin ctypes layer over it and `synth` builds the seeded synthetic workloads.
The HIP library is loaded lazily on first use and its absence is an error: there is
no CPU fallback.
"""
__all__ = ["binding", "synth", "build"]
