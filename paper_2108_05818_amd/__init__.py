"""psx: chunked mixed-precision Adam for MI355X (gfx950) behind a C-ABI library.

`paper_2108_05818_amd.psx` is the thin ctypes binding of include/psx.h;
`paper_2108_05818_amd.workloads` holds the seeded synthetic workloads.
The native library is loaded on first use and its absence is an error: there
is no CPU fallback.
"""
__all__ = ["psx", "workloads"]
