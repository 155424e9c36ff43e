"""pQuant decoupled linear layer for MI355X (gfx950): HIP kernels behind a C-ABI library.

Importing the package loads nothing; `paper_2602_22592_amd.binding` loads libpquant.so on first use
and raises if it has not been built (there is no CPU fallback).
"""
__all__ = ["workloads", "binding", "build"]
