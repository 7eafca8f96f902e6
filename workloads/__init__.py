"""Seeded synthetic inputs (shared by the CPU oracle's tests and the HIP path's tests and bench)."""
from . import rng, layers  # noqa: F401
from .layers import LayerSpec  # noqa: F401
