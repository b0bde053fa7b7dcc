"""libchunkft: the ChunkFT hot path (chunk-restricted weight gradient + chunk
AdamW + cycle planner) as hand-written gfx950 kernels behind a C ABI.

`binding` holds the ctypes wrappers (same names as the C entry points);
`workloads` the seeded synthetic inputs; `build` compiles the library.
Nothing is loaded at import time.
"""

__all__ = ["binding", "workloads", "build"]
