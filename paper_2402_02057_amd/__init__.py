"""MI355X-native lookahead-step attention and greedy verification (arXiv 2402.02057).

`paper_2402_02057_amd.binding` is the thin ctypes layer over the C-ABI HIP library;
`paper_2402_02057_amd.workloads` holds the seeded synthetic input generators;
`paper_2402_02057_amd.lookahead` is the host side of a decoding run (window, n-gram pool).  Importing
this package loads nothing: the HIP library is opened on the first call into the binding
and a missing library is an error, never a fallback.
"""
__all__ = ["binding", "workloads", "buildlib", "lookahead"]
