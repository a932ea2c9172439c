"""Pins for the CPU oracle: checks against things other than the oracle itself.

Each `pin_*` function takes `lib` (None = the built oracle, or the path of an
alternative build) and raises AssertionError when the oracle under test
violates what the paper's definition (section 3.2.1: softmax attention over
the sink + recent set) or plain mathematics fixes.  test_oracle_pins.py runs
them on the real oracle; test_oracle_mutants.py runs them on deliberately
broken copies and requires that each copy is caught.
"""
import math
import os

import numpy as np
import torch

import oracle
from workloads import make_custom, poison_unretained

PAGE = 128
D = 576
DV = 512
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def run(inp, lib=None, **kw):
    return oracle.oracle_decode(inp.q, inp.kv_cache, inp.kv_scales, inp.page_table,
                                inp.seq_lens_host, inp.sink, inp.window, inp.softmax_scale,
                                kv_dtype=inp.kv_dtype, lib=lib, **kw)


# ---------------------------------------------------------------- helpers ---
def explicit_index_list(L, S, W):
    """The retained set written as an explicit de-duplicated list (second
    equation of 3.2.1 shifted to 0-based, both ranges clipped to [0, L))."""
    sink = list(range(0, min(S, L)))
    recent = list(range(max(L - W, 0), L))
    return sorted(set(sink) | set(recent))


def rows_f64(inp, b, positions):
    """Independent gather: logical positions -> fp64 rows via torch indexing and
    torch's own bf16 / float8 widening."""
    pos = torch.as_tensor(positions, dtype=torch.long)
    pages = inp.page_table.cpu()[b].long()[pos // PAGE]
    flat = pages * PAGE + (pos % PAGE)
    cache = inp.kv_cache.cpu().reshape(-1, D)
    rows = cache[flat].to(torch.float32).to(torch.float64)
    if inp.kv_dtype == "fp8":
        sc = inp.kv_scales.cpu().reshape(-1)[flat].to(torch.float64)
        rows = rows * sc[:, None]
    return rows


def library_attention(inp, b, positions):
    """softmax(q K^T scale) V with torch library routines in fp64 -> (out [H,512], lse [H])."""
    H = inp.heads
    if len(positions) == 0:
        return torch.zeros(H, DV, dtype=torch.float64), torch.full((H,), -math.inf, dtype=torch.float64)
    rows = rows_f64(inp, b, positions)
    q = inp.q.cpu()[b].to(torch.float64)
    scale = float(np.float32(inp.softmax_scale))
    logits = (q @ rows.T) * scale
    p = torch.softmax(logits, dim=-1)
    return p @ rows[:, :DV], torch.logsumexp(logits, dim=-1)


def set_row(inp, b, j, vec):
    """Write a full 576-vector (exactly representable values) at logical position j."""
    page = int(inp.page_table[b, j // PAGE])
    inp.kv_cache[page, j % PAGE] = torch.as_tensor(vec, dtype=torch.float32).to(inp.kv_cache.dtype)


def close(a, b, tol, what):
    a = np.asarray(a, dtype=np.float64)
    b = np.broadcast_to(np.asarray(b, dtype=np.float64), a.shape)
    with np.errstate(invalid="ignore"):
        d = np.abs(a - b)
    d = np.where((a == b) | (np.isnan(a) & np.isnan(b)), 0.0, d)   # equal infinities, matching NaNs
    err = np.max(d) if a.size else 0.0
    assert np.array_equal(np.isnan(a), np.isnan(b)) and not (err > tol), f"{what}: max abs err {err} > {tol}"


# ------------------------------------------------------------------- pins ---
def pin_decoders(lib=None):
    """Storage decoders against torch's own widening, all codes, plus values
    fixed by the formats' definitions."""
    L = oracle.binding._load(lib) if lib else oracle.binding._load()
    codes = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    ref = codes.view(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([L.oracle_bf16_to_double(i) for i in range(65536)])
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    ok = ~np.isnan(ref)
    assert np.array_equal(got[ok], ref[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(ref[ok]))

    c8 = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    ref8 = c8.view(torch.float8_e4m3fn).to(torch.float32).to(torch.float64).numpy()
    got8 = np.array([L.oracle_fp8_e4m3_to_double(i) for i in range(256)])
    assert np.array_equal(np.isnan(got8), np.isnan(ref8))
    ok = ~np.isnan(ref8)
    assert np.array_equal(got8[ok], ref8[ok])
    # OCP E4M3 fixed points: max finite, one, smallest normal / subnormal, NaN codes
    assert got8[0x7E] == 448.0 and got8[0xFE] == -448.0
    assert got8[0x38] == 1.0 and got8[0x08] == 2.0 ** -6 and got8[0x01] == 2.0 ** -9
    assert got8[0x00] == 0.0 and math.isnan(got8[0x7F]) and math.isnan(got8[0xFF])
    assert got8[0x78] == 256.0  # e=15, m=0 is finite in E4M3 (no infinities)


def pin_retained_predicate(lib=None):
    L_ = oracle.binding._load(lib) if lib else oracle.binding._load()
    for L in range(0, 41):
        for S in range(0, L + 3):
            for W in range(0, L + 3):
                got = [j for j in range(-2, L + 3) if L_.oracle_is_retained(j, L, S, W)]
                assert got == explicit_index_list(L, S, W), (L, S, W)


def pin_worked_example(lib=None):
    vals = {}
    with open(os.path.join(GOLDEN, "two_token_worked_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    inp = make_custom(1, 1, [5], 1, 1, shuffled_pages=False, seed=1, softmax_scale=1.0)
    inp.q.zero_()
    inp.q[0, 0, 0] = 1.0
    for j in range(5):
        row = np.zeros(D)
        row[0] = {0: 0.0, 4: 1.0}.get(j, 8.0)
        row[1] = j + 1
        set_row(inp, 0, j, row)
    out, lse, probs = run(inp, lib, want_probs=True)
    close(probs[0, 0, 0], vals["p0"], 1e-15, "p0")
    close(probs[0, 0, 4], vals["p4"], 1e-15, "p4")
    close(probs[0, 0, 1:4], 0.0, 0.0, "unretained weights")
    close(out[0, 0, 0], vals["out0"], 1e-15, "out0")
    close(out[0, 0, 1], vals["out1"], 1e-14, "out1")
    close(out[0, 0, 2:], 0.0, 0.0, "other dims")
    close(lse[0, 0], vals["lse"], 1e-15, "lse")


def pin_dense_reduction(lib=None, kv_dtype="bf16"):
    """S + W >= L: every position kept once; equals library dense attention."""
    lens = [300, 129, 1, 257]
    for (S, W) in [(0, 400), (128, 300), (300, 0), (64, 236), (300, 300)]:
        inp = make_custom(4, 3, lens, S, W, seed=11, kv_dtype=kv_dtype,
                          q_std=1.0, kv_std=(1.0 if kv_dtype == "fp8" else 0.5),
                          spare_pages=2)
        out, lse = run(inp, lib)
        for b, L in enumerate(lens):
            keep = list(range(L)) if S + W >= L else explicit_index_list(L, S, W)
            ro, rl = library_attention(inp, b, keep)
            close(out[b], ro, 1e-12, f"dense out b={b} S={S} W={W}")
            close(lse[b], rl, 1e-12, f"dense lse b={b}")


def pin_bruteforce_tiny(lib=None):
    """All (S, W) for small L against library attention on the explicit list."""
    rng = np.random.default_rng(5)
    for L in [0, 1, 2, 7, 19]:
        inp = make_custom(2, 2, [L, max(L - 1, 0)], 0, 0, seed=100 + L, q_std=2.0, kv_std=1.0)
        for S in range(0, L + 3):
            for W in range(0, L + 3):
                inp.sink, inp.window = S, W
                out, lse = run(inp, lib)
                for b, Lb in enumerate(inp.seq_lens_host):
                    ro, rl = library_attention(inp, b, explicit_index_list(Lb, S, W))
                    close(out[b], ro, 1e-12, f"L={Lb} S={S} W={W} out")
                    close(lse[b], rl, 1e-12, f"L={Lb} S={S} W={W} lse")
    # sparse, multi-page, unaligned
    for (Lb, S, W) in [(1000, 37, 200), (513, 128, 129), (2048, 64, 512), (700, 0, 5), (700, 9, 0)]:
        inp = make_custom(1, 2, [Lb], S, W, seed=int(rng.integers(1 << 30)), q_std=3.0, kv_std=1.0)
        out, lse = run(inp, lib)
        ro, rl = library_attention(inp, 0, explicit_index_list(Lb, S, W))
        close(out[0], ro, 1e-12, f"sparse L={Lb} out")
        close(lse[0], rl, 1e-12, f"sparse L={Lb} lse")


def pin_softmax_invariants(lib=None):
    inp = make_custom(2, 4, [900, 300], 50, 130, seed=3, q_std=4.0, kv_std=1.0)
    out, lse, probs = run(inp, lib, want_probs=True)
    scale = float(np.float32(inp.softmax_scale))
    for b, L in enumerate(inp.seq_lens_host):
        keep = explicit_index_list(L, inp.sink, inp.window)
        mask = np.zeros(probs.shape[-1], bool)
        mask[keep] = True
        rows = rows_f64(inp, b, keep).numpy()
        for h in range(inp.heads):
            p = probs[b, h]
            assert np.all(p >= 0) and np.all(p[~mask] == 0)
            assert abs(p.sum() - 1.0) < 1e-12
            assert np.all(out[b, h] <= rows[:, :DV].max(0) + 1e-12)
            assert np.all(out[b, h] >= rows[:, :DV].min(0) - 1e-12)
            s = scale * rows @ inp.q[b, h].to(torch.float64).numpy()
            assert s.max() - 1e-12 <= lse[b, h] <= s.max() + math.log(len(keep)) + 1e-12
            # weights reproduce exp(s - lse)
            close(p[keep], np.exp(s - lse[b, h]), 1e-12, "p = exp(s - lse)")


def pin_page_permutation(lib=None):
    """Same logical content under two different physical page orders -> same bits."""
    a = make_custom(3, 2, [640, 130, 1025], 100, 260, seed=21, q_std=2.0, kv_std=1.0, spare_pages=3)
    out_a, lse_a = run(a, lib)
    g = torch.Generator().manual_seed(99)
    perm = torch.randperm(a.num_pages, generator=g)          # new physical id of old page i
    b = make_custom(3, 2, [640, 130, 1025], 100, 260, seed=21, q_std=2.0, kv_std=1.0, spare_pages=3)
    b.kv_cache[perm] = a.kv_cache.clone()
    tab = a.page_table.clone()
    valid = tab >= 0
    tab[valid] = perm[tab[valid].long()].to(torch.int32)
    b.page_table = tab
    out_b, lse_b = run(b, lib)
    assert np.array_equal(out_a, out_b) and np.array_equal(lse_a, lse_b)


def pin_poison(lib=None, kv_dtype="bf16"):
    """NaN in every slot outside the retained set (and in unreferenced pages) changes nothing."""
    lens = [1000, 77, 400]
    S, W = 40, 150
    inp = make_custom(3, 2, lens, S, W, seed=8, kv_dtype=kv_dtype, q_std=2.0, kv_std=1.0, spare_pages=4)
    out0, lse0 = run(inp, lib)
    keep = []
    for L in lens:
        n = ((L + PAGE - 1) // PAGE) * PAGE
        kept = set(explicit_index_list(L, S, W))
        keep.append([j in kept for j in range(n)])
    poison_unretained(inp, keep)
    assert torch.isnan(inp.kv_cache.float()).any()
    out1, lse1 = run(inp, lib)
    assert not np.isnan(out1).any() and not np.isnan(lse1).any()
    assert np.array_equal(out0, out1) and np.array_equal(lse0, lse1)
    # a NaN inside the retained set must propagate (row 0 is a sink of sequence 0)
    page = int(inp.page_table[0, 0])
    if kv_dtype == "bf16":
        inp.kv_cache[page, 0, 5] = float("nan")
    else:
        inp.kv_cache.view(torch.uint8)[page, 0, 5] = 0x7F
    out2, _ = run(inp, lib)
    assert np.isnan(out2[0]).all() and not np.isnan(out2[1:]).any()


def pin_closed_forms(lib=None):
    L, S, W = 500, 30, 70
    keep = explicit_index_list(L, S, W)
    N = len(keep)
    scale = float(np.float32(192.0 ** -0.5))
    rng = np.random.default_rng(0)

    # (i) identical keys -> uniform weights: out = their common value part, lse = s + ln N
    inp = make_custom(1, 3, [L], S, W, seed=1, q_std=1.0, kv_std=1.0)
    krow = torch.randn(D, generator=torch.Generator().manual_seed(4)).to(torch.bfloat16)
    for j in keep:
        set_row(inp, 0, j, krow.float())
    out, lse, probs = run(inp, lib, want_probs=True)
    close(probs[0][:, keep], 1.0 / N, 1e-15, "uniform weights")
    close(out[0], np.tile(krow.double().numpy()[:DV], (3, 1)), 1e-12, "identical rows out")
    s = scale * (inp.q[0].double() @ krow.double()).numpy()
    close(lse[0], s + math.log(N), 1e-12, "identical rows lse")

    # (ii) q = 0 -> uniform: out = mean of retained values, lse = ln N
    inp = make_custom(1, 2, [L], S, W, seed=2, q_std=1.0, kv_std=1.0)
    inp.q.zero_()
    out, lse = run(inp, lib)
    close(out[0, 0], rows_f64(inp, 0, keep)[:, :DV].mean(0).numpy(), 1e-12, "q=0 mean")
    close(lse[0], math.log(N), 1e-13, "q=0 lse")

    # (iii) identical value parts, different rope parts -> out = that value for any q
    inp = make_custom(1, 2, [L], S, W, seed=3, q_std=3.0, kv_std=1.0)
    vrow = torch.randn(DV, generator=torch.Generator().manual_seed(6)).to(torch.bfloat16)
    for j in keep:
        page = int(inp.page_table[0, j // PAGE])
        inp.kv_cache[page, j % PAGE, :DV] = vrow
    # make logits vary through the rope dims only (q's first 512 dims still hit vrow equally)
    out, lse = run(inp, lib)
    close(out[0], np.tile(vrow.double().numpy(), (2, 1)), 1e-12, "equal values out")

    # (iv) one dominating key -> out -> its value, lse -> its logit
    inp = make_custom(1, 1, [L], S, W, seed=4, q_std=1.0 / 24, kv_std=1.0 / 24)
    jstar = keep[N // 2]
    inp.q.zero_()
    inp.q[0, 0, 520] = 64.0                      # a rope dim: does not touch the values
    big = rows_f64(inp, 0, [jstar])[0].clone()
    big[520] = 16.0                              # logit = 64*16*scale ~ 73.9
    set_row(inp, 0, jstar, big.float())
    out, lse = run(inp, lib)
    close(out[0, 0], rows_f64(inp, 0, [jstar])[0, :DV].numpy(), 1e-12, "spike out")
    close(lse[0, 0], 64.0 * 16.0 * scale, 1e-10, "spike lse")

    # (v) shift every retained key by delta living in rope dims: lse moves by scale*q.delta, out unchanged
    inp = make_custom(1, 2, [L], S, W, seed=5, q_std=1.0, kv_std=0.25)
    # quarter-integers in rope dims keep key + delta exactly representable in bf16
    for j in keep:
        page = int(inp.page_table[0, j // PAGE])
        r = rng.integers(-8, 9, size=64) / 4.0
        inp.kv_cache[page, j % PAGE, DV:] = torch.as_tensor(r, dtype=torch.float32).to(torch.bfloat16)
    out_a, lse_a = run(inp, lib)
    delta = np.zeros(D)
    delta[DV:] = rng.integers(-4, 5, size=64) / 2.0
    for j in keep:
        set_row(inp, 0, j, rows_f64(inp, 0, [j])[0].numpy() + delta)
    out_b, lse_b = run(inp, lib)
    c = scale * (inp.q[0].double().numpy() @ delta)
    close(lse_b[0] - lse_a[0], c, 1e-11, "shift lse")
    close(out_b, out_a, 1e-12, "shift out")


def pin_merge_identity(lib=None):
    """Disjoint sink and recent ranges: the whole equals the lse-weighted merge
    of a sink-only call and a recent-only call."""
    lens = [900, 400]
    S, W = 70, 200
    inp = make_custom(2, 3, lens, S, W, seed=13, q_std=3.0, kv_std=1.0)
    out, lse = run(inp, lib)
    inp.sink, inp.window = S, 0
    out_s, lse_s = run(inp, lib)
    inp.sink, inp.window = 0, W
    out_w, lse_w = run(inp, lib)
    tot = np.logaddexp(lse_s, lse_w)
    merged = np.exp(lse_s - tot)[..., None] * out_s + np.exp(lse_w - tot)[..., None] * out_w
    close(lse, tot, 1e-12, "merge lse")
    close(out, merged, 1e-12, "merge out")


def pin_boundary_spikes(lib=None):
    """A single huge-logit token placed next to each edge of the retained set
    must count exactly when the definition says so."""
    L, S, W = 1000, 130, 260
    scale = float(np.float32(192.0 ** -0.5))
    cases = {0: True, S - 1: True, S: False, L - W - 1: False, L - W: True, L - 1: True,
             (S + L - W) // 2: False}
    for j, counted in cases.items():
        inp = make_custom(1, 1, [L], S, W, seed=17, q_std=1.0 / 24, kv_std=1.0 / 24)
        inp.q.zero_()
        inp.q[0, 0, 530] = 64.0
        row = np.zeros(D)
        row[530] = 16.0
        row[7] = 3.0
        set_row(inp, 0, j, row)
        out, lse = run(inp, lib)
        if counted:
            close(out[0, 0, 7], 3.0, 1e-9, f"spike at {j} must count")
            close(lse[0, 0], 1024.0 * scale, 1e-9, f"spike lse at {j}")
        else:
            assert abs(out[0, 0, 7]) < 0.1 and lse[0, 0] < 10.0, f"spike at {j} must not count"
    # window longer than the sequence, sink longer than the sequence, empty set
    inp = make_custom(3, 1, [5, 0, 3], 0, 0, seed=2, q_std=1.0, kv_std=1.0)
    out, lse = run(inp, lib)
    assert np.all(out == 0) and np.all(np.isneginf(lse))


def pin_scale_and_value_slice(lib=None):
    """The scale multiplies the logits (not the output) and values are dims
    0..511 only: checked through lse's closed form for two tokens and an
    output that must ignore the rope dims."""
    inp = make_custom(1, 1, [2], 2, 0, seed=1, shuffled_pages=False, softmax_scale=0.25)
    inp.q.zero_()
    inp.q[0, 0, 3] = 2.0
    r0 = np.zeros(D); r0[3] = 4.0; r0[0] = 1.0; r0[511] = -2.0; r0[512] = 100.0
    r1 = np.zeros(D); r1[3] = -4.0; r1[0] = 3.0; r1[511] = 6.0; r1[575] = 100.0
    set_row(inp, 0, 0, r0)
    set_row(inp, 0, 1, r1)
    out, lse, probs = run(inp, lib, want_probs=True)
    # logits: 0.25 * 2 * (+-4) = +-2  -> p0 = 1/(1+e^-4)
    p0 = 1.0 / (1.0 + math.exp(-4.0))
    close(probs[0, 0, 0], p0, 1e-15, "p0")
    close(lse[0, 0], 2.0 + math.log1p(math.exp(-4.0)), 1e-14, "lse")
    close(out[0, 0, 0], p0 * 1.0 + (1 - p0) * 3.0, 1e-14, "out dim 0")
    close(out[0, 0, 511], p0 * -2.0 + (1 - p0) * 6.0, 1e-14, "out dim 511")
    assert out.shape[-1] == DV


def pin_multi_query(lib=None):
    """Several causal queries per sequence: the rows of query t must equal plain library
    attention over the explicit position list of a sequence cut after that query's token."""
    import copy
    rng = np.random.default_rng(5)
    for T in (2, 3, 4):
        Hq = 3
        lens = [T, T + 1, 37, 130, 261]
        for S, W in ((0, 5), (3, 0), (2, 7), (40, 100), (128, 140), (1000, 1000)):
            inp = make_custom(len(lens), T * Hq, lens, S, W, seed=int(rng.integers(1 << 30)),
                              q_std=1.0, kv_std=1.0)
            out, lse = run(inp, lib, q_len=T)
            for b, L in enumerate(lens):
                for t in range(T):
                    Lt = L - (T - 1 - t)          # keys 0 .. Lt-1 are visible to query t
                    positions = explicit_index_list(Lt, S, W)
                    view = copy.copy(inp)
                    view.q = inp.q[:, t * Hq:(t + 1) * Hq]
                    ref_o, ref_l = library_attention(view, b, positions)
                    close(out[b, t * Hq:(t + 1) * Hq], ref_o.numpy(), 1e-11, f"mq out T={T} b={b} t={t}")
                    close(lse[b, t * Hq:(t + 1) * Hq], ref_l.numpy(), 1e-11, f"mq lse T={T} b={b} t={t}")


def pin_fp8(lib=None):
    pin_dense_reduction(lib, kv_dtype="fp8")
    pin_poison(lib, kv_dtype="fp8")
    # sparse fp8 against the library on explicit lists
    inp = make_custom(2, 2, [700, 333], 33, 190, seed=31, kv_dtype="fp8", q_std=0.2, kv_std=1.0)
    out, lse = run(inp, lib)
    for b, L in enumerate(inp.seq_lens_host):
        ro, rl = library_attention(inp, b, explicit_index_list(L, 33, 190))
        close(out[b], ro, 1e-12, "fp8 sparse out")
        close(lse[b], rl, 1e-12, "fp8 sparse lse")


ALL_PINS = [pin_decoders, pin_retained_predicate, pin_worked_example, pin_dense_reduction,
            pin_bruteforce_tiny, pin_softmax_invariants, pin_page_permutation, pin_poison,
            pin_closed_forms, pin_merge_identity, pin_boundary_spikes,
            pin_scale_and_value_slice, pin_multi_query, pin_fp8]
