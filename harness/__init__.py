"""Seeded synthetic inputs shared by the CPU oracle tests and the GPU path.

This package holds no arithmetic of the method itself: it only draws Q/K/V
and plants the three attention structures the paper names.
"""
