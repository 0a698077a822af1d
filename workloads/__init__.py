"""Seeded synthetic inputs and graph descriptions shared by the oracle-side and the
GPU-side harnesses.  This package holds no arithmetic of the method: it only *describes*
expressions (as data) and draws random tensors."""
from .graphspec import GraphSpec  # noqa: F401
