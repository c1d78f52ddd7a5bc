"""Speculative Thinking hot path on MI355X: HIP kernels behind a C-ABI library plus a thin binding.

`binding` loads the built shared library and fails loudly when it is missing; `synth` holds the
seeded input generators; `cost` holds the closed-form byte / FLOP counts used for rooflines.
"""
