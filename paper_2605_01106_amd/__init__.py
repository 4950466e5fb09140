"""Component-aware self-speculative decoding hot path for parallel-hybrid
(Mamba-2 + attention) decoders on MI355X.

``workloads`` draws the seeded synthetic inputs; ``binding`` is the thin ctypes
layer over the C-ABI library (``libhh.so``, built from ``csrc/``); ``build``
compiles it.  Importing ``binding`` fails loudly when the library is missing.
"""
from . import workloads  # noqa: F401
