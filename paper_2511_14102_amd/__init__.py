"""MI355X-native MoE draft/verify layer for MoE-SpeQ-style speculative quantized decoding.

`binding` is the thin ctypes layer over libmoespeq.so (argument marshalling only; every step of
the path runs in the HIP kernels), `pack` builds the kernel-native weight layouts."""
from . import pack  # noqa: F401
from .binding import (  # noqa: F401
    MoeError, LayerDesc, Context, load_library, library_path,
    MOE_VERIFY_ACCUMULATE, MOE_VERIFY_ONLY_LISTED, MOE_VERIFY_STRICT,
)
