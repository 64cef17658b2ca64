"""MorphKV decode hot path for MI355X: C-ABI library (csrc/, include/morphkv.h) and its ctypes binding."""
from . import inputs  # noqa: F401  (seeded generators; no GPU needed)

__all__ = ["inputs", "binding", "build"]
