"""MI355X-native decode hot path of LaRoSA (layerwise rotated sparse activation).

Sub-modules:
  synth    seeded synthetic inputs (no method arithmetic)
  api      thin ctypes binding over liblarosa.so (argument marshalling only)
  prepare  offline preparation (PCA rotation, weight folding) with torch
The HIP library is loaded on first use of `api`; a missing library raises.
"""
__all__ = ["synth"]
