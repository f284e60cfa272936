"""Multi-token paged attention and KV append for MI355X (gfx950).

Thin Python binding over the C-ABI library ``libpv.so`` (hand-written HIP).
Importing this package does not load the library; ``paper_2312_05516_amd.binding``
does, and fails loudly if it has not been built.
"""

__all__ = ["workloads"]
