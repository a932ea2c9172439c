"""fp64 CPU oracle for sparse MLA decode (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It shares no code with the HIP library.
"""
from .binding import (  # noqa: F401
    build,
    oracle_decode,
    bf16_to_double,
    fp8_e4m3_to_double,
    is_retained,
    lib_path,
)
