"""The approximation of section 3.2.1 (attention over the kept set ~ dense attention) on inputs
with planted sink and recency mass: the distance to dense attention shrinks as S and W grow,
vanishes when everything is kept, and the lse gap equals -log of the kept softmax mass, which
the oracle's weights give independently."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_22481_amd.approx_error import sweep
from workloads import make_planted


@pytest.mark.gpu
def test_error_shrinks_with_the_kept_set_and_matches_the_kept_mass():
    ctx = 3000
    inp = make_planted(2, 16, ctx, seed=3, device="cuda:0")
    settings = [(0, 64), (4, 64), (4, 512), (4, 1500), (128, 1500), (128, ctx)]
    rows = sweep(inp, settings)
    rel = [r["rel_l2_vs_dense"] for r in rows]
    assert rel[0] > rel[1] > rel[2] > rel[3] >= rel[4] > rel[5]      # sinks matter, then the window
    assert rows[-1]["rel_l2_vs_dense"] <= 1e-6 and abs(rows[-1]["max_lse_gap"]) <= 1e-5
    assert rel[0] > 0.05 and rel[3] < 0.05
    # kept softmax mass from the oracle's dense weights, summed over the kept positions
    _, _, probs = oracle.oracle_decode(inp.q, inp.kv_cache, inp.kv_scales, inp.page_table,
                                       inp.seq_lens_host, 0, ctx, inp.softmax_scale, want_probs=True)
    for r in rows[:-1]:
        S, W = r["sink"], r["window"]
        keep = np.zeros(ctx, dtype=bool)
        keep[:S] = True
        keep[ctx - W:] = True
        mass = probs[..., keep].sum(-1)
        assert abs(mass.min() - r["min_kept_mass"]) <= 2e-3 * mass.min() + 1e-6, (r, mass.min())
