"""MI355X-native hot path of BOF4 / BOF4-S / OPQ 4-bit block-wise weight quantisation (arxiv 2505.06653).

The compute lives in csrc/ (hand-written HIP for gfx950 behind a C ABI, declared in include/bof4.h); `binding`
marshals torch device pointers into that ABI.  Importing the package does not load the library; the first call
does, and fails loudly if it has not been built (python -m paper_2505_06653_amd.build).
"""
from . import codebooks, inputs  # noqa: F401

__all__ = ["codebooks", "inputs", "binding", "build"]
