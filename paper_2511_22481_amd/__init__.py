"""MI355X-native sparse MLA decode over the OmniAttn retained set.

Thin ctypes binding over libomniattn.so (hand-written gfx950 HIP kernels behind
the C ABI in include/omniattn.h).  There is no CPU fallback: without the built
library, or without a GPU, plan/decode raise.
"""
from .binding import (  # noqa: F401
    OmniAttnError,
    Plan,
    Problem,
    omniattn_plan,
    omniattn_plan_host,
    omniattn_plan_update,
    omniattn_decode,
    omniattn_decode_timed,
    omniattn_decode_static,
    omniattn_static_scratch_bytes,
    omniattn_ring_pages,
    omniattn_ring_slot,
    omniattn_ring_append,
    decode,
    lib_path,
    load_library,
    BF16,
    FP8_E4M3,
    FP32,
)
