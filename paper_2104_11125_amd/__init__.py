"""ScaleCom's per-step compression path (CLT-k with low-pass-filtered error feedback,
arXiv 2104.11125, Alg. 1) as hand-written HIP kernels for gfx950 behind a small C-ABI.

``paper_2104_11125_amd.binding`` is the thin Python layer over that C-ABI (it needs the
built library and raises if it is missing); ``paper_2104_11125_amd.workloads`` holds the
seeded synthetic inputs.
"""
