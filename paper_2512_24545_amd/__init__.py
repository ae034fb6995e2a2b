"""MI355X-native forward product for Multi-Envelope Double Binary Factorization (MDBF).

The package holds the HIP/C-ABI library sources (csrc/), a thin ctypes binding
(binding.py, loaded lazily) and the seeded input generators (synth.py).
"""

__all__ = ["binding", "synth"]
