"""CPU oracle for fusion groups (test infrastructure; see interp.py)."""
from .interp import run  # noqa: F401
