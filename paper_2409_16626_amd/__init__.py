"""HiF8 (HiFloat8) conversion kernels for AMD MI355X.

`paper_2409_16626_amd.hif8` is the binding over the C-ABI library libhif8.so
(hand-written HIP kernels for gfx950); `paper_2409_16626_amd.workloads` holds the
seeded synthetic input generators.  Nothing here falls back to a CPU path.
"""
