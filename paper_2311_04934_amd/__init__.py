"""MI355X-native Prompt Cache hot path (arXiv 2311.04934): module pool, KV assembly,
RoPE at schema positions and uncached-token prefill attention, as hand-written
gfx950 HIP kernels behind a C ABI (``include/promptcache.h``).

``binding`` is the ctypes face of the shared library; ``workloads`` describes
seeded synthetic inputs.  Importing this package loads nothing native; the
library is opened on first use and its absence is an error, never a fallback.
"""
__all__ = ["binding", "workloads"]
