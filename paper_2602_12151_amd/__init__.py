"""MI355X-native paged GQA decode attention for heterogeneous (mixed-length) batches.

`workloads` draws the seeded synthetic inputs; `binding` is the thin ctypes
layer over the C-ABI library built from `csrc/` (imported on first use so that
input generation works on machines without the built library).
"""
__all__ = ["workloads", "binding"]
