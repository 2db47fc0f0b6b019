"""MI355X-native reranker scoring over cached document KV (HyperRAG hot path).

Sub-modules are imported on demand so that the seeded input generators
(`workloads`) can be used without loading the HIP library, and the HIP
binding (`binding`) without touching anything else.
"""

__all__ = ["workloads", "binding", "build"]
