"""CPU-only checks of the C ABI: the library loads, exports every symbol the header
declares, validates arguments, and the host planner's tiles and segments cover
exactly the retained set (paper section 3.2.1, second equation)."""
import ctypes
import os
import random
import re

import pytest

import paper_2511_22481_amd as oa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "omniattn.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(omniattn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = oa.load_library()
    names = declared_functions()
    assert "omniattn_plan" in names and "omniattn_decode" in names and len(names) >= 15
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/omniattn.h but not exported"


def retained_set(L, S, W):
    # literal predicate, written here independently of the library and of the oracle
    return [j for j in range(L) if j < S or j >= L - W]


def plan_for(lens, S, W, H=128, cus=256, hint=0):
    mp = max(1, max((L + 127) // 128 for L in lens))
    return oa.omniattn_plan_host(lens, num_cus=cus, batch=len(lens), num_heads=H,
                                 max_pages_per_seq=mp, num_pages=max(1, sum((L + 127) // 128 for L in lens)),
                                 sink=S, window=W, softmax_scale=0.1, num_splits_hint=hint)


def check_plan(lens, S, W, H=128, cus=256, hint=0):
    plan = plan_for(lens, S, W, H, cus, hint)
    T = plan.tile_tokens
    assert 128 % T == 0
    segs = plan.segments()
    assert len(segs) == plan.num_segments
    n_hb = (H + plan.head_block - 1) // plan.head_block
    total = 0
    for b, L in enumerate(lens):
        R = retained_set(L, S, W)
        total += len(R)
        for hb in range(n_hb):
            mine = [s for s in segs if s["b"] == b and s["hb"] == hb]
            assert mine, (b, hb)
            nt = mine[0]["ntiles"]
            # segments partition [0, ntiles) in order, without gaps or overlap
            mine.sort(key=lambda s: s["tile_lo"])
            pos = 0
            for s in mine:
                assert s["L"] == L and s["ntiles"] == nt
                assert s["tile_lo"] == pos and s["tile_hi"] >= s["tile_lo"]
                pos = s["tile_hi"]
            assert pos == nt
            if len(mine) > 1:
                assert all(s["slot"] >= 0 for s in mine)
            else:
                assert mine[0]["slot"] == -1
            # the tiles cover every retained position exactly once and nothing else needs reading
            covered = []
            for t in range(nt):
                lo, hi = plan.tile_range(b, t)
                assert lo % T == 0 and hi == lo + T
                assert lo // 128 == (hi - 1) // 128, "a tile must not straddle a page"
                inside = [j for j in range(lo, min(hi, L)) if j < S or j >= L - W]
                assert inside, f"tile {t} of sequence {b} holds no retained position"
                covered += inside
            assert covered == R, (b, L, S, W)
    assert plan.retained_tokens == total
    slots = sorted(s["slot"] for s in segs if s["slot"] >= 0)
    assert slots == list(range(plan.num_partials))
    units = sorted(set(s["unit"] for s in segs))
    assert units == list(range(plan.num_units))
    want_ws = plan.num_partials * plan.head_block * (4 + 512 * 2)     # fp32 lse + bf16 row
    assert want_ws <= plan.workspace_bytes < want_ws + 512
    return plan


def test_plan_covers_retained_set_exhaustive_small():
    for L in list(range(0, 70)) + [127, 128, 129, 255, 256, 257]:
        for S in (0, 1, 31, 32, 33, 64, 100, 300):
            for W in (0, 1, 31, 32, 33, 64, 129, 300):
                check_plan([L], S, W, H=16, cus=4)


def test_plan_random_batches():
    rng = random.Random(7)
    for _ in range(60):
        B = rng.randint(1, 9)
        lens = [rng.choice([0, 1, rng.randint(1, 5000)]) for _ in range(B)]
        S = rng.choice([0, 5, 64, 128, 1000])
        W = rng.choice([0, 7, 512, 2048, 9000])
        H = rng.choice([1, 16, 48, 128, 160])
        hint = rng.choice([0, 0, 1, 2, 3, 7, 1000])
        check_plan(lens, S, W, H=H, cus=rng.choice([1, 8, 256]), hint=hint)


def test_plan_headline_shapes():
    p = check_plan([32768] * 64, 128, 2048)
    assert p.retained_tokens == 64 * 2176
    assert p.num_units <= 256 and p.head_block == 128
    p = check_plan([4096] * 32, 128, 8192)          # S + W >= L: everything retained
    assert p.retained_tokens == 32 * 4096
    p = check_plan([131072] * 32, 128, 8192)
    assert p.retained_tokens == 32 * 8320


def test_split_hint_cuts_every_sequence():
    p = plan_for([32 * 40] * 3, 0, 1 << 20, hint=7)
    assert p.max_splits == 7 and p.num_partials == 21 and p.num_units == 21 and p.head_block == 128
    p = plan_for([32 * 2] * 3, 0, 1 << 20, hint=7)   # fewer tiles than pieces
    assert p.max_splits == 2
    p = plan_for([32 * 40] * 3, 0, 1 << 20, hint=1)
    assert p.max_splits == 1 and p.num_partials == 0 and p.workspace_bytes == 0


def test_plan_update_equals_fresh_plan():
    """Planning again into an existing object (every decode step changes every length) gives
    the plan a fresh omniattn_plan_host call gives, segment by segment."""
    rng = random.Random(11)
    for _ in range(25):
        B = rng.randint(1, 12)
        S = rng.choice([0, 64, 128])
        W = rng.choice([0, 512, 2048, 9000])
        H = rng.choice([16, 128, 160])
        cus = rng.choice([8, 256])
        hint = rng.choice([0, 0, 3])
        lens = [rng.randint(1, 6000) for _ in range(B)]
        mp = 64
        kw = dict(num_cus=cus, batch=B, num_heads=H, max_pages_per_seq=mp, num_pages=B * mp,
                  sink=S, window=W, softmax_scale=0.1, num_splits_hint=hint)
        plan = oa.omniattn_plan_host(lens, **kw)
        for step in range(4):
            lens = [min(L + rng.choice([1, 1, 1, 200]), mp * 128) for L in lens]
            oa.omniattn_plan_update(plan, lens)
            fresh = oa.omniattn_plan_host(lens, **kw)
            assert plan.segments() == fresh.segments()
            for name in ("num_units", "num_partials", "max_splits", "num_splits", "retained_tokens",
                         "workspace_bytes"):
                assert getattr(plan, name) == getattr(fresh, name), name
        # a rejected length leaves the plan as it was
        before = plan.segments()
        with pytest.raises(oa.OmniAttnError):
            oa.omniattn_plan_update(plan, [mp * 128 + 1] * B)
        assert plan.segments() == before


def test_argument_validation():
    ok = dict(batch=1, num_heads=16, max_pages_per_seq=4, num_pages=4, sink=1, window=1,
              softmax_scale=1.0)
    oa.omniattn_plan_host([10], **ok)
    bad = [dict(ok, batch=0), dict(ok, num_heads=0), dict(ok, sink=-1), dict(ok, window=-1),
           dict(ok, max_pages_per_seq=0), dict(ok, num_pages=0), dict(ok, num_splits_hint=-1),
           dict(ok, softmax_scale=float("nan"))]
    for kw in bad:
        with pytest.raises(oa.OmniAttnError) as e:
            oa.omniattn_plan_host([10], **kw)
        assert e.value.code == -1, kw
    for kw in [dict(ok, qk_dim=512), dict(ok, v_dim=576), dict(ok, page_size=64),
               dict(ok, kv_dtype=7), dict(ok, out_dtype=oa.FP8_E4M3)]:
        with pytest.raises(oa.OmniAttnError) as e:
            oa.omniattn_plan_host([10], **kw)
        assert e.value.code == -2, kw
    with pytest.raises(oa.OmniAttnError):            # more pages than the table row holds
        oa.omniattn_plan_host([4 * 128 + 1], **ok)
    with pytest.raises(oa.OmniAttnError):            # negative length
        oa.omniattn_plan_host([-1], **ok)


def test_null_pointers_and_host_plan_cannot_decode():
    lib = oa.load_library()
    assert lib.omniattn_plan_host(None, None, None, 1) == -1
    h = ctypes.c_void_p()
    assert lib.omniattn_plan_host(ctypes.byref(h), None, None, 1) == -1 and not h.value
    plan = oa.omniattn_plan_host([10], batch=1, num_heads=16, max_pages_per_seq=1, num_pages=1,
                                 sink=1, window=1, softmax_scale=1.0)
    one = ctypes.c_void_p(0x1000)
    rc = lib.omniattn_decode(plan.handle, one, one, None, one, one, one, None, 0, None)
    assert rc == -1                                   # a host-only plan has no device metadata
    assert lib.omniattn_decode(None, one, one, None, one, one, one, None, 0, None) == -1
    lib.omniattn_plan_destroy(None)                   # allowed
    assert lib.omniattn_strerror(-3).decode().startswith("workspace")
    assert lib.omniattn_strerror(12345).decode() == "unknown error code"


def test_no_cpu_fallback():
    """Without a GPU the product path must fail loudly, never compute on the CPU."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(oa.OmniAttnError) as e:
        oa.omniattn_plan([10], batch=1, num_heads=16, max_pages_per_seq=1, num_pages=1, sink=1,
                         window=1, softmax_scale=1.0)
    assert e.value.code == -4
    q = torch.zeros(1, 16, 576, dtype=torch.bfloat16)
    kv = torch.zeros(1, 128, 576, dtype=torch.bfloat16)
    with pytest.raises(oa.OmniAttnError):
        oa.decode(q, kv, None, torch.zeros(1, 1, dtype=torch.int32), [10], 1, 1, 1.0)


def test_product_never_imports_oracle():
    pkg = os.path.join(ROOT, "paper_2511_22481_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
