"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU harness.

This module holds NONE of the method's arithmetic: only a counter-based Gaussian
generator that gives bit-identical fp32 values on the host (numpy, synth.gen) and on
the device (synth/fill.hip, loaded by synth.fill), so that both sides of a parity test
start from the same initial state, the same c_i and the same per-event gradient noise.
"""
