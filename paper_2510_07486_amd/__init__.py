"""MI355X-native KV-selection hot path of AsyncSpade (predict -> score -> top-k -> sparse attention).

`api` is the ctypes binding of the C-ABI HIP library; `workloads` draws seeded synthetic inputs;
`build` compiles the library for gfx950.
"""
from . import workloads  # noqa: F401

__all__ = ["api", "workloads", "build"]
