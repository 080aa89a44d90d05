"""Fused gradient-reduce + Adam/LAMB step for one GPU's parameter shard on MI355X (gfx950).

`binding` is the thin ctypes layer over the C-ABI library; `workloads` holds the seeded synthetic
inputs.  Nothing is loaded at import time; the first call into `binding` loads libccfused.so and
raises if it is missing.
"""
__all__ = ["binding", "workloads"]
