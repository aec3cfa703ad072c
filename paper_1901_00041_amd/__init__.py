"""Fused multi-tenant convolution ("super-kernel") for MI355X / gfx950.

`synth` (seeded workloads, numpy only) can be imported anywhere.  The binding (`st_conv`) loads the
HIP shared library on first use and fails loudly if it has not been built.
"""
__all__ = ["synth", "st_conv"]
