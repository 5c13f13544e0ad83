"""Seeded synthetic safetensors inputs (structure, writer, procedural byte source).

Shared by the CPU oracle's tests and the GPU path's tests; holds none of the method's arithmetic.
"""
