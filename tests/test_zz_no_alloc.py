"""omniattn_decode_static (no workspace argument, library-owned device scratch) against
omniattn_decode: same kernels, same plan, so the results must be bitwise equal.  Two calls
in a row, the second on a smaller input, so that stale partial rows of the first call sit
in the shared scratch buffer when the second runs."""
import pytest
import torch

import paper_2511_22481_amd as oa
from workloads import make_custom

from parity import assert_parity, to_device

pytestmark = pytest.mark.gpu


def _both(inp, hint):
    plan = oa.omniattn_plan(inp.seq_lens_host, batch=inp.batch, num_heads=inp.heads,
                            max_pages_per_seq=inp.max_pages, num_pages=inp.num_pages,
                            sink=inp.sink, window=inp.window, softmax_scale=inp.softmax_scale,
                            kv_dtype=oa.FP8_E4M3 if inp.kv_dtype == "fp8" else oa.BF16,
                            out_dtype=oa.BF16, num_splits_hint=hint)
    assert plan.num_partials > 0, "the case must use the scratch buffer"
    assert plan.workspace_bytes <= oa.omniattn_static_scratch_bytes()
    dev = inp.q.device
    out_a = torch.full((inp.batch, inp.heads, 512), float("nan"), dtype=torch.bfloat16, device=dev)
    lse_a = torch.full((inp.batch, inp.heads), float("nan"), dtype=torch.float32, device=dev)
    out_b, lse_b = out_a.clone(), lse_a.clone()
    ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device=dev)
    oa.omniattn_decode(plan, inp.q, inp.kv_cache, inp.kv_scales, inp.page_table, out_a, lse_a, ws)
    oa.omniattn_decode_static(plan, inp.q, inp.kv_cache, inp.kv_scales, inp.page_table, out_b, lse_b)
    torch.cuda.synchronize()
    assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16))
    assert torch.equal(lse_a.view(torch.int32), lse_b.view(torch.int32))
    return out_b, lse_b


def test_static_scratch_matches_workspace_path_twice():
    big = to_device(make_custom(batch=6, heads=128, seq_lens=[5000, 4097, 3000, 2500, 777, 4500],
                                sink=128, window=2048, seed=71))
    out, lse = _both(big, hint=4)
    assert_parity(big, out, lse, what="static scratch, first call")
    small = to_device(make_custom(batch=2, heads=48, seq_lens=[900, 1300], sink=64, window=512,
                                  seed=72, kv_dtype="fp8"))
    out, lse = _both(small, hint=3)
    assert_parity(small, out, lse, what="static scratch, second (smaller) call")


def test_static_scratch_rejects_oversized_plan():
    # 96 sequences cut four ways with 128 heads: 384 partial slots of 128 KiB exceed 40 MiB
    inp = to_device(make_custom(batch=96, heads=128, seq_lens=[1024] * 96, sink=0, window=1024, seed=73))
    plan = oa.omniattn_plan(inp.seq_lens_host, batch=inp.batch, num_heads=inp.heads,
                            max_pages_per_seq=inp.max_pages, num_pages=inp.num_pages,
                            sink=inp.sink, window=inp.window, softmax_scale=inp.softmax_scale,
                            kv_dtype=oa.BF16, out_dtype=oa.BF16, num_splits_hint=4)
    assert plan.workspace_bytes > oa.omniattn_static_scratch_bytes()
    out = torch.empty((inp.batch, inp.heads, 512), dtype=torch.bfloat16, device=inp.q.device)
    lse = torch.empty((inp.batch, inp.heads), dtype=torch.float32, device=inp.q.device)
    with pytest.raises(oa.OmniAttnError) as ei:
        oa.omniattn_decode_static(plan, inp.q, inp.kv_cache, inp.kv_scales, inp.page_table, out, lse)
    assert ei.value.code == -6
