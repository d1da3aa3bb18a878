"""MI355X-native pack -> ragged attention -> unpack (hand-written HIP for gfx950 behind a C ABI).

Importing the package loads nothing; ``paper_2604_15408_amd.binding`` opens the shared library on
first use and raises if it has not been built (there is no CPU fallback).
"""

__all__ = ["binding", "build", "workloads"]
