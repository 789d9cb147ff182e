"""MI355X-native hot path of dynamic-weighted elastic AdaHessian (Xu & Carr, arXiv 2409.09242).

`workloads` holds the seeded synthetic inputs; `binding` is the thin ctypes layer over the C-ABI
library built from `csrc/` (it raises if the library has not been built).
"""
