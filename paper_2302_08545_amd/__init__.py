"""THC (Tensor Homomorphic Compression, arXiv 2302.08545) hot path for AMD MI355X (gfx950).

`paper_2302_08545_amd.api` is a thin ctypes binding over the C-ABI in include/thc.h;
`paper_2302_08545_amd.workloads` holds the seeded synthetic gradient generators.
Nothing is loaded at import time; the HIP library is opened on first use and there is no
CPU fallback: a missing library raises.
"""
__all__ = ["api", "workloads", "build"]
