"""ROAST hashing hot path for MI355X (gfx950): ROAST-MM forward / dX / dM and the hashed-chunk
embedding lookup, as hand-written HIP kernels behind a C-ABI library.

`paper_2207_10702_amd.binding` exposes the library's entry points under the same names
(argument marshalling only); `paper_2207_10702_amd.workloads` draws the seeded synthetic inputs.
"""
__all__ = ["binding", "workloads", "build"]
