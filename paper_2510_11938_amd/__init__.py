"""flexstage: MI355X-native forward step of one pipeline stage (a contiguous
decoder-layer range over a ragged batch with a paged KV cache) and the KV-cache
repartition used when stage boundaries are merged or split at run time.

``paper_2510_11938_amd.binding`` is the thin ctypes layer over the C-ABI library
(``include/flexstage.h``); ``paper_2510_11938_amd.synth`` draws the seeded
synthetic workloads.  Importing this package loads nothing native; the library
is opened on first use and a missing build is an error, never a fallback.
"""
__all__ = ["binding", "synth", "build"]
