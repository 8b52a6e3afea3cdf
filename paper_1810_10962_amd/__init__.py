"""libbns: sampled batch normalisation (Batch Normalization Sampling, arXiv 1810.10962) for MI355X.

The compute lives in ``libbns.so`` (hand-written HIP for gfx950, C ABI declared in
``include/bns.h``); ``paper_1810_10962_amd.bns`` is a thin ctypes binding with the same
names.  Importing this package does not load the shared library; the binding does,
and raises if it is missing.  There is no CPU fallback.
"""
