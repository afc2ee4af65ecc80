"""SWA + learnable token eviction (LTE) token mixer for MI355X (gfx950).

The compute lives in hand-written HIP kernels behind the C ABI declared in
include/ltea.h; `paper_2510_20787_amd.binding` marshals arguments to it.
Importing this package does not load the shared library; the first call does,
and fails loudly if it has not been built.
"""
__all__ = ["workloads", "binding"]
