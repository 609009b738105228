"""Seeded synthetic input generators shared by the CPU oracle and the GPU tests."""
from . import synth  # noqa: F401
