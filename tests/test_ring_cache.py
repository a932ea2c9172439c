"""Physically compressed cache (sink pages pinned, recent pages in a ring).

CPU: the page mapping the library exports is simulated token by token and checked
against the literal retained predicate: at every length, every retained position's
logical page must still sit in the page it was written to.
GPU: tokens are appended one at a time to a ring cache (library kernel) and to a full
cache (plain indexing); decoding either must give bitwise the same result, and that
result must match the oracle run on the full cache.
"""
import numpy as np
import pytest
import torch

import paper_2511_22481_amd as oa
import parity
from workloads.generate import Inputs, quantize_fp8_per_token

PAGE = 128


def retained(j, L, S, W):
    return 0 <= j < L and (j < S or j >= L - W)


@pytest.mark.parametrize("S,W", [(0, 1), (1, 0), (0, 0), (100, 130), (128, 256), (129, 1), (300, 700),
                                 (64, 128), (5, 127), (256, 129)])
def test_ring_mapping_never_loses_a_retained_token(S, W):
    n_pages = oa.omniattn_ring_pages(S, W)
    assert n_pages == (S + PAGE - 1) // PAGE + (W + PAGE - 1) // PAGE + 1
    holds = {}                      # own page index -> logical page it currently holds
    for L_before in range(0, 9 * PAGE + 37):
        lp = L_before // PAGE
        slot = oa.omniattn_ring_slot(S, W, lp)
        assert 0 <= slot < n_pages
        if L_before % PAGE == 0:
            holds[slot] = lp        # the new token opens logical page lp
        assert holds[slot] == lp
        L = L_before + 1
        for j in range(L):
            if retained(j, L, S, W):
                assert holds.get(oa.omniattn_ring_slot(S, W, j // PAGE)) == j // PAGE, (L, j)
    assert oa.omniattn_ring_slot(S, W, -1) == -1 and oa.omniattn_ring_pages(-1, 3) == -1


@pytest.mark.parametrize("T", [2, 3, 64])
@pytest.mark.parametrize("S,W", [(0, 128), (0, 1), (100, 130), (128, 256), (64, 127), (5, 129)])
def test_ring_mapping_with_several_queries(S, W, T):
    """T queries per decode call: query t sees a sequence of length L - (T - 1 - t) and keeps
    its own sinks and window, so the earliest one reaches T - 1 tokens further back.  The ring
    sized for q_len = T must hold every position any of the T queries keeps, at every length."""
    n_pages = oa.omniattn_ring_pages(S, W, q_len=T)
    assert n_pages == oa.omniattn_ring_pages(S, W + T - 1)
    holds = {}
    for L_before in range(0, 7 * PAGE + 11):
        lp = L_before // PAGE
        slot = oa.omniattn_ring_slot(S, W, lp, q_len=T)
        assert 0 <= slot < n_pages
        if L_before % PAGE == 0:
            holds[slot] = lp
        assert holds[slot] == lp
        L = L_before + 1
        if L < T:
            continue
        for t in (0, T // 2, T - 1):
            Lq = L - (T - 1 - t)
            # every page of the two retained ranges (both ends and one position per page between)
            lo = max(Lq - W, 0)
            js = set(range(0, min(S, Lq), PAGE)) | set(range(lo, Lq, PAGE)) | {min(S, Lq) - 1, lo, Lq - 1}
            for j in js:
                if retained(j, Lq, S, W):
                    assert holds.get(oa.omniattn_ring_slot(S, W, j // PAGE, q_len=T)) == j // PAGE, (L, t, j)


def test_ring_sized_for_one_query_loses_tokens_of_three():
    """The case that motivates the rule above: S = 0, W = 128, three queries, L = 257.  Query 0
    keeps token 127, whose page a ring laid out for one query has already handed on."""
    S, W, T, L = 0, 128, 3, 257
    lost = []
    for sized_for in (1, T):
        holds = {}
        for pos in range(L):
            if pos % PAGE == 0:
                holds[oa.omniattn_ring_slot(S, W, pos // PAGE, q_len=sized_for)] = pos // PAGE
        j = L - (T - 1) - W      # first position query 0 keeps
        lost.append(holds.get(oa.omniattn_ring_slot(S, W, j // PAGE, q_len=sized_for)) != j // PAGE)
    assert lost == [True, False]


def _decode(q, cache, scales, table, lens, S, W, scale):
    out, lse, _ = oa.decode(q, cache, scales, table, lens, S, W, scale)
    torch.cuda.synchronize()
    return out, lse


@pytest.mark.gpu
@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_ring_cache_decodes_like_the_full_cache(kv_dtype):
    dev = torch.device("cuda:0")
    g = torch.Generator(device="cpu").manual_seed(31)
    B, H, S, W, T = 5, 48, 70, 300, 1100
    scale = 1.0 / np.sqrt(192.0)
    fp8 = kv_dtype == "fp8"
    max_pages = (T + PAGE - 1) // PAGE + 1
    ring_pages = oa.omniattn_ring_pages(S, W)
    cdtype = torch.float8_e4m3fn if fp8 else torch.bfloat16

    def empty_pool(n):
        c = torch.zeros((n, PAGE, 576), dtype=torch.float32, device=dev).to(cdtype)
        sc = torch.ones((n, PAGE), dtype=torch.float32, device=dev) if fp8 else None
        return c, sc

    # full cache: every logical page has its own page
    full, full_sc = empty_pool(B * max_pages)
    full_tab = torch.randperm(B * max_pages, generator=g).to(torch.int32).reshape(B, max_pages).to(dev)
    # ring cache: each sequence owns ring_pages pages of a small pool; unread entries are garbage
    ring, ring_sc = empty_pool(B * ring_pages + 3)
    seq_pages = torch.randperm(B * ring_pages + 3, generator=g)[:B * ring_pages].to(torch.int32)
    seq_pages = seq_pages.reshape(B, ring_pages).to(dev)
    ring_tab = torch.full((B, max_pages), -7, dtype=torch.int32, device=dev)
    lens_dev = torch.zeros(B, dtype=torch.int32, device=dev)
    rows_all = (torch.randn((T, B, 576), generator=g) * 0.5)
    q = (torch.randn((B, H, 576), generator=g) * 0.3).to(torch.bfloat16).to(dev)

    checkpoints = {1, 69, 70, 71, 127, 128, 129, 370, 371, 500, 640, 897, T}
    for t in range(T):
        if fp8:
            codes, sc = quantize_fp8_per_token(rows_all[t])
            new_rows, new_sc = codes.to(dev), sc.to(dev)
        else:
            new_rows, new_sc = rows_all[t].to(torch.bfloat16).to(dev), None
        # full cache by plain indexing
        phys = full_tab[:, t // PAGE].long()
        full[phys, t % PAGE] = new_rows
        if fp8:
            full_sc[phys, t % PAGE] = new_sc
        # ring cache by the library
        oa.omniattn_ring_append(lens_dev, new_rows, new_sc, seq_pages, ring, ring_sc, ring_tab,
                                sink=S, window=W)
        L = t + 1
        if L in checkpoints:
            assert lens_dev.tolist() == [L] * B
            lens = [L] * B
            out_f, lse_f = _decode(q, full, full_sc, full_tab, lens, S, W, scale)
            out_r, lse_r = _decode(q, ring, ring_sc, ring_tab, lens, S, W, scale)
            assert torch.equal(out_f, out_r) and torch.equal(lse_f, lse_r), L
    # the last state against the oracle (on the full cache: the plain logical view)
    inp = Inputs(q=q, kv_cache=full, kv_scales=full_sc, page_table=full_tab,
                 seq_lens=torch.tensor([T] * B, dtype=torch.int32), seq_lens_host=[T] * B, sink=S,
                 window=W, softmax_scale=scale, kv_dtype=kv_dtype)
    parity.assert_parity(inp, out_r, lse_r, row_rel_l2=2e-2, what="ring cache " + kv_dtype)
    # the oracle on the ring view (its unread page-table entries are garbage) sees the same
    # logical cache: identical fp64 results
    ring_inp = Inputs(q=q, kv_cache=ring, kv_scales=ring_sc, page_table=ring_tab,
                      seq_lens=inp.seq_lens, seq_lens_host=[T] * B, sink=S, window=W,
                      softmax_scale=scale, kv_dtype=kv_dtype)
    ro_f, rl_f = parity.run_oracle(inp)
    ro_r, rl_r = parity.run_oracle(ring_inp)
    assert np.array_equal(ro_f, ro_r) and np.array_equal(rl_f, rl_r)
    # a full sequence is left alone
    lens_dev.fill_(max_pages * PAGE)
    before = ring.clone()
    oa.omniattn_ring_append(lens_dev, new_rows, new_sc, seq_pages, ring, ring_sc, ring_tab, sink=S, window=W)
    torch.cuda.synchronize()
    assert lens_dev.tolist() == [max_pages * PAGE] * B and torch.equal(before.view(torch.uint8), ring.view(torch.uint8))
