"""MI355X-native SlideSparse linear layer: (2N-2):2N sparse weights run on 2:4 sparse MFMA.

The compute lives in libslidesparse.so (hand-written HIP for gfx950, C ABI declared in
include/slidesparse.h); `binding` marshals torch device tensors into it."""
from . import synth  # noqa: F401  (pure numpy; safe without a GPU)

__all__ = ["synth", "binding", "build"]
