"""Natural GaLore optimizer step for MI355X (gfx950): HIP kernels behind a C ABI.

``binding`` is the thin ctypes layer over the shared library (it raises if the
library has not been built); ``workloads`` holds the seeded synthetic inputs.
"""
__all__ = ["binding", "workloads"]
