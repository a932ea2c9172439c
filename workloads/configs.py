"""The five decode workloads, as plain records.

Shapes follow the DeepSeek-R1 absorbed-MLA decode layout: each cached token is
one latent row of 576 values (512 compressed-KV dims then 64 rope dims); the
value of a token is the first 512 of those.  `sink` and `window` are the
N_sink / N_recent hyper-parameters of the retained set (paper section 3.2.1,
second equation).  The paper gives no numeric values for them, nor context
lengths; these records fix them.
"""
from dataclasses import dataclass, replace
import math

QK_DIM = 576
V_DIM = 512
PAGE = 128


@dataclass(frozen=True)
class Config:
    name: str
    batch: int
    heads: int
    sink: int
    window: int
    # fixed context length, or (lo, hi) for lengths uniform in [lo, hi] inclusive
    ctx: object
    kv_dtype: str = "bf16"          # "bf16" | "fp8"
    shuffled_pages: bool = True     # False = identity page table (contiguous cache)
    kv_std: float = 1.0 / math.sqrt(QK_DIM)
    q_std: float = 1.0 / math.sqrt(QK_DIM)
    softmax_scale: float = 1.0 / math.sqrt(192.0)
    seed: int = 20251122
    poison_tail: bool = False       # NaN in slots >= L_b of the last page

    def scaled(self, **kw):
        return replace(self, **kw)


CONFIGS = {
    # tiny: the oracle finishes in well under a second
    "tiny": Config("tiny", batch=4, heads=16, sink=64, window=512, ctx=2048,
                   shuffled_pages=False, seed=20251122),
    # DeepSeek-R1-shaped decode, the headline workload
    "r1_b64_32k": Config("r1_b64_32k", batch=64, heads=128, sink=128, window=2048,
                         ctx=32768, seed=20251123),
    # mixed lengths, exercises split-KV + combine
    "mixed_b256": Config("mixed_b256", batch=256, heads=128, sink=128, window=4096,
                         ctx=(1024, 65536), seed=20251124, poison_tail=True),
    # every position retained: must equal dense attention
    "dense_b32_4k": Config("dense_b32_4k", batch=32, heads=128, sink=128, window=8192,
                           ctx=4096, seed=20251125),
    # the headline shape with nothing compressed (a layer the pattern search leaves dense):
    # every one of the 32768 positions is retained
    "r1_b64_32k_dense": Config("r1_b64_32k_dense", batch=64, heads=128, sink=0, window=32768,
                               ctx=32768, seed=20251127),
    # long context, fp8 e4m3 cache with one fp32 scale per token
    "fp8_b32_128k": Config("fp8_b32_128k", batch=32, heads=128, sink=128, window=8192,
                           ctx=131072, kv_dtype="fp8", kv_std=1.0, seed=20251126),
}


def get_config(name: str) -> Config:
    return CONFIGS[name]
