"""Seeded synthetic inputs (no distance arithmetic lives here)."""
from . import synth  # noqa: F401
