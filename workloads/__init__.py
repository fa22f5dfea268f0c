"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

Nothing in this package performs any step of the rounding method: it only draws
random tensors with the shapes and statistics of LLM linear layers.
"""
