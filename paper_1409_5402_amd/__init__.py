"""MI355X-native SAME Gibbs LDA sweep: HIP kernels behind a C-ABI library, plus a thin binding.

Importing the package loads nothing native; :mod:`paper_1409_5402_amd.binding` loads the
built library on first use and raises if it is missing (there is no CPU fallback).
"""
__all__ = ["binding", "schedule", "synth"]
