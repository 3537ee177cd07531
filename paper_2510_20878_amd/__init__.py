"""MI355X-native hotness-aware mixed-precision KV-chunk load (HA-RAG hot path).

`binding`    ctypes view of the C-ABI library built from csrc/ (include/ha_rag.h)
`workloads`  seeded synthetic inputs
`build`      compiles csrc/ for gfx950 into lib/libha_rag.so
"""
__all__ = ["binding", "workloads", "build"]
