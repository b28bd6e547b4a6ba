"""libnatcomp for MI355X: natural compression and natural dithering of fp32 gradients
(arXiv 1905.10988) as hand-written gfx950 HIP kernels behind a C ABI.

`natcomp`   ctypes binding of the C ABI (argument marshalling only).
`workloads` seeded synthetic gradients shaped like the paper's workloads.
"""
