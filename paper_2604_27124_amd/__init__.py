"""MI355X-native padded bidirectional sigmoid attention (forward and backward).

The compute lives in the HIP library ``libsigattn.so`` behind a C ABI
(``include/sigmoid_attn.h``); this package is the thin Python binding over it
plus the seeded workload generator.  Nothing here falls back to a CPU path: the
binding raises if the library is missing.
"""

__all__ = ["binding", "workloads"]
