"""MI355X-native hot path of Polymorph: context selection and the multi-LoRA ViT forward.

``synth`` holds the seeded input generators; ``binding`` is the thin ctypes
layer over the C-ABI library built from ``csrc/`` (it raises if the library is
missing: there is no CPU fallback).
"""
