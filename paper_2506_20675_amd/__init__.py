"""MI355X-native MoE verification path for utility-driven speculative decoding.

`binding` wraps the C-ABI library (HIP kernels for gfx950 + the host-side policy);
`synth` is the seeded synthetic-input generator used by tests and the benchmark.
Importing this package loads nothing; the shared library is opened on first use and
its absence is an error (there is no CPU fallback).
"""
