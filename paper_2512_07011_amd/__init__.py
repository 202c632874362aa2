"""Block-Sparse FlashAttention forward (prefill) for MI355X (gfx950).

The product is the C-ABI library ``libbsfa.so`` built from ``csrc/``; ``binding`` is a thin
ctypes layer over it and ``synth`` holds the seeded input recipes.  Nothing is loaded at
import time: the library is opened on the first call and a missing build raises.
"""

__all__ = ["binding", "synth"]
