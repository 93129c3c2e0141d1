"""MI355X-native decode hot path of LaRoSA (layerwise rotated sparse activation).

Sub-modules:
  synth    seeded synthetic inputs (no method arithmetic)
  api      thin ctypes binding over liblarosa.so (argument marshalling only)
  offline  the offline part driven through the library (second moments, folding, adapters; eigen-solver by torch)
  allocation  kept counts K1..K4 from sparsity and the App. B coefficients (host bookkeeping)
The HIP library is loaded on first use of `api`; a missing library raises.
"""
__all__ = ["synth"]
