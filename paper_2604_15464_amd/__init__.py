"""MI355X-native ragged paged attention (fused KV-cache update + causal GQA
attention over a ragged mixed batch).  The compute path lives in the HIP
library built from csrc/; `rpa` is its ctypes binding and is imported lazily
so that the input generators can be used without the library."""

__all__ = ["workloads"]
