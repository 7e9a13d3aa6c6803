"""MI355X-native ADSA decode path (hand-written HIP for gfx950) and its Python binding.

Submodules: `binding` (ctypes mirror of include/adsa.h), `batch` (device-memory plumbing),
`build` (hipcc build of the library), `workloads` (seeded synthetic inputs).
Nothing here falls back to a CPU implementation: without the built library every call raises.
"""
__all__ = ["binding", "batch", "build", "workloads"]
