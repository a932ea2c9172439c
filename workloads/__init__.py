"""Seeded synthetic inputs for sparse MLA decode.

This package only draws random tensors and lays them out in pages; it holds
none of the attention arithmetic and is the single module shared by the HIP
tests, the benchmark and the CPU oracle's tests.
"""
from .configs import CONFIGS, Config, get_config  # noqa: F401
from .generate import (  # noqa: F401
    Inputs,
    make_inputs,
    make_custom,
    make_planted,
    quantize_fp8_per_token,
    poison_unretained,
)
