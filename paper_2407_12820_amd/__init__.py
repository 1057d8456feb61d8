"""MI355X-native decode hot path of PQ-based KV-cache retrieval (PQCache, arxiv 2407.12820).

Sub-modules:
  workloads  seeded synthetic inputs (no method arithmetic)
  build      compiles csrc/*.hip into libpqcache.so for gfx950
  binding    ctypes marshalling over the C ABI declared in include/pqcache.h

Nothing here imports the CPU oracle, and importing this package does not load the
HIP library; `binding` does, and fails loudly when it is missing.
"""

__all__ = ["workloads", "build", "binding"]
