"""Batched forward evaluation of recursive tree networks on one MI355X.

`binding` mirrors the C ABI of include/treelstm.h (the HIP library is loaded on first
use and there is no fallback); `synth` draws the seeded synthetic inputs.
"""
