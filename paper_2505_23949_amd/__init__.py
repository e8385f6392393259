"""MI355X-native transposable N:M mask finder (TSENOR hot path).

``binding`` holds the ctypes binding of the C-ABI library (``include/tsenor.h``),
``synth`` the seeded synthetic workloads, ``build`` the hipcc build step.
Nothing is loaded at import time; ``binding.load()`` raises if the HIP library
has not been built - there is no CPU fallback.
"""
__all__ = ["binding", "synth", "build"]
