"""LightTransfer hot path for one MI355X: thin Python binding over the C-ABI library.

Importing this package loads nothing; the first call into `lt` loads liblt_hip.so and raises
if it is missing and cannot be built.  There is no CPU fallback.
"""
from . import lt  # noqa: F401

__all__ = ["lt"]
