"""MI355X-native table-batched embedding forward + fused sparse backward with moment-scaled row-wise AdaGrad.

The arithmetic lives in libtbe355.so (hand-written HIP for gfx950, C ABI declared in include/tbe355.h);
`binding` only marshals torch device tensors into that ABI."""
from .binding import (TBE, TbeError, lib_path, load_library, EXPORTS)  # noqa: F401
