"""MI355X-native MoE expert module (router, permutation, grouped SwiGLU FFN, combine).

The hot path is the HIP library built from csrc/ behind the C ABI of include/moe.h;
`binding` is a ctypes layer over it.  Importing this package does not load the library.
"""
from .binding import Moe, MoeError, MoeShape, make_shape, shape_of, workspace_bytes, h_scratch_bytes, load_library, estimate_streamed_ms, STAGES  # noqa: F401
