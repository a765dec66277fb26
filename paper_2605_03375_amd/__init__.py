"""MI355X-native per-layer KV object path (pack / unpack / submission entries) of arxiv 2605.03375.

`binding` holds the ctypes binding of libtutti (the HIP library); `workloads` the seeded
synthetic inputs.  Importing the package loads nothing; `binding.lib()` raises if the HIP
library has not been built.
"""
__all__ = ["binding", "workloads", "build", "placement"]
