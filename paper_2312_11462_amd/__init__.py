"""MI355X-native verify path of Cascade Speculative Drafting (hand-written HIP, gfx950).

The product is the C-ABI library `libcsd.so` declared in include/csd.h; this package is a
thin ctypes binding over it (argument marshalling only) plus the build step.  PyTorch is used
for device memory and streams, nothing else.  There is no CPU fallback: without the built
library, or without a GPU, the calls raise.
"""
from .binding import (CsdError, Model, accept, bigram_draft, bigram_draft_append, bigram_fit, cascade_gate, maxgram_draft, tree_accept, debug_copy, debug_mfma, debug_read, lib,  # noqa: F401
                      library_path,
                      EXPORTS)
