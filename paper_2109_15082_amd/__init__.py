"""MI355X-native MREM module step (Algorithm 2 of the paper) behind a C-ABI.

`synth` holds the seeded input generators; `binding` is the ctypes layer over
the HIP library (imported on demand: it raises if the library is not built).
"""
__all__ = ["synth", "binding"]
