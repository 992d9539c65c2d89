"""XOR-friendly binary quantized top-K cosine search for MI355X (gfx950).

The product is the C-ABI library ``libxbq.so`` (HIP kernels + host launchers,
declared in ``include/xbq.h``); :mod:`paper_2008_02002_amd.xbq` is the thin ctypes
binding over it.  Importing the package does not load the library; the first call
into the binding does, and fails loudly if it has not been built.
"""
__all__ = ["xbq", "workloads"]
