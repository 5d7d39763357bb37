"""MI355X-native bit-packed merged-expert MoE FFN (PuzzleMoE inference hot path).

``synth`` draws the seeded synthetic workloads; ``binding`` is the thin ctypes layer
over the HIP C-ABI library (loaded lazily, fails loudly if it is not built).
"""
__all__ = ["synth", "binding"]
