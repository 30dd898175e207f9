"""MI355X-native bidirectional Mamba mixer path (conv + SiLU, bidirectional selective scan, gate, combine).

Importing the package loads nothing; `paper_2511_15927_amd.binding` loads the HIP library on first use
and raises if it has not been built (there is no CPU fallback).
"""
__all__ = ["synth", "binding", "shapes"]
