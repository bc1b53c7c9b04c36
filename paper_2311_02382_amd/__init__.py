"""MI355X-native segment attention for sequence-parallel transformers.

The hot path of the LSS Transformer (Section 3, Principle 3, Eq. 2): the
partial self-attention of one sequence segment, forward and backward, as
hand-written HIP kernels for gfx950 behind a C-ABI library.  ``lss`` is the
thin binding over that library; ``synth`` draws the seeded inputs.

Nothing is loaded at import time; the first call into ``lss`` loads the built
library and fails loudly if it is missing.
"""
__all__ = ["lss", "synth"]
