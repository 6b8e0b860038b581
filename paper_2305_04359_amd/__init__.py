"""MI355X-native Vamana graph build (prefix-doubling batch insertion) and beam search.

`binding` wraps the C ABI of include/ann.h; `workloads` draws the synthetic inputs; `build`
compiles the HIP sources.  Importing this package loads nothing heavy.
"""
__all__ = ["binding", "workloads", "build"]
