"""Segmented / full sum-reduction and inclusive scan of fp16 data on MI355X (gfx950).

The compute path is the HIP library built from ``csrc/`` and reached through the
C ABI declared in ``include/tcr.h``; ``binding`` marshals arguments only.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads"]
