"""Seeded random sweep over the decode's options at small sizes: batch, heads, lengths (empty,
one token, page and tile edges), sink / window, cache type, output type, forced splits, several
queries, poison in every slot outside the kept set.  Every case is compared element by element
with the oracle through the C ABI (paper section 3.2.1)."""
import numpy as np
import pytest
import torch

import paper_2511_22481_amd as oa
import oracle
import parity
from workloads import make_custom, poison_unretained

pytestmark = pytest.mark.gpu
PAGE = 128


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    T = int(rng.choice([1, 1, 1, 2, 3]))
    H = int(rng.choice([16, 32, 48, 64, 128]))
    B = int(rng.integers(1, 7))
    edges = [0, 1, 2, 31, 32, 33, 127, 128, 129, 255, 256, 257, 1000, 2047, 2049, 3500]
    lens = [int(rng.choice(edges)) if rng.random() < 0.6 else int(rng.integers(1, 3000)) for _ in range(B)]
    lens = [L if L == 0 or L >= T else T for L in lens]
    S = int(rng.choice([0, 1, 31, 32, 64, 100, 128, 130, 4000]))
    W = int(rng.choice([0, 1, 32, 33, 100, 128, 257, 1000, 4000]))
    return dict(T=T, H=H, B=B, lens=lens, S=S, W=W,
                kv_dtype=str(rng.choice(["bf16", "fp8"])),
                out_fp32=bool(rng.random() < 0.3),
                hint=int(rng.choice([0, 0, 1, 2, 3, 7])),
                poison=bool(rng.random() < 0.5),
                q_std=float(rng.choice([1.0 / 24, 0.5, 1.5])))


@pytest.mark.parametrize("seed", range(32))
def test_random_case(seed):
    c = _case(seed)
    T, H, B, lens, S, W = c["T"], c["H"], c["B"], c["lens"], c["S"], c["W"]
    inp = parity.to_device(make_custom(B, T * H, lens, S, W, seed=seed, kv_dtype=c["kv_dtype"],
                                       q_std=c["q_std"], kv_std=1.0 if c["kv_dtype"] == "fp8" else 0.7,
                                       spare_pages=2))
    if c["poison"]:
        # kept by at least one of the T queries: query t sees a sequence of length L - (T - 1 - t)
        keep = []
        for L in lens:
            n = ((L + PAGE - 1) // PAGE) * PAGE
            keep.append([any(j < Lq and (j < S or j >= Lq - W) for Lq in range(max(L - T + 1, 0), L + 1) if Lq > 0)
                         for j in range(n)])
        poison_unretained(inp, keep)
    q = inp.q.reshape(B, T, H, 576) if T > 1 else inp.q
    out, lse, plan = oa.decode(q, inp.kv_cache, inp.kv_scales, inp.page_table, inp.seq_lens_host, S, W,
                               inp.softmax_scale, out_dtype=torch.float32 if c["out_fp32"] else None,
                               num_splits_hint=c["hint"])
    torch.cuda.synchronize()
    out = out.reshape(B, T * H, 512)
    lse = lse.reshape(B, T * H)
    ref_o, ref_l = oracle.oracle_decode(inp.q, inp.kv_cache, inp.kv_scales, inp.page_table, inp.seq_lens_host,
                                        S, W, inp.softmax_scale, kv_dtype=inp.kv_dtype, q_len=T)
    e = parity.errors(out, lse, ref_o, ref_l)
    assert e["max_abs"] <= parity.MAX_ABS * parity.abs_scale(out, ref_o, inp.kv_dtype), (c, e)
    assert e["rel_l2"] <= parity.REL_L2[inp.kv_dtype], (c, e)
    assert e["lse_abs"] <= parity.LSE_ABS, (c, e)
    assert e["worst_row_rel_l2"] <= (parity.FP8_ROW_REL_L2 if inp.kv_dtype == "fp8" else 1e-2), (c, e)
