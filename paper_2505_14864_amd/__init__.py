"""MI355X-native token-routed sparse FFN layer (DynMo hot path).

`workloads` draws the seeded synthetic inputs; `binding` is the thin ctypes
layer over the C-ABI library built from `csrc/` (it raises if the library has
not been built -- there is no CPU fallback).
"""
