"""MI355X-native query-aware page selection + sparse decode attention (TinyServe hot path).

`paper_2509_12211_amd.tinyserve` is the thin ctypes binding over the C-ABI HIP
library (include/tinyserve.h); `paper_2509_12211_amd.workloads` generates the
seeded synthetic inputs.  There is no CPU fallback: the binding raises if the
HIP library has not been built.
"""
__all__ = ["tinyserve", "workloads"]
