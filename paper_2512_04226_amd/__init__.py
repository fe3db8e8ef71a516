"""MI355X-native GEMM with an analytical kernel selector (arXiv 2512.04226's method).

`binding` mirrors the C ABI of include/gemm.h; `api.matmul` is the one-call convenience over it
(cached analytic selection, workspace kept per device); `workloads` generates the seeded inputs.
"""
