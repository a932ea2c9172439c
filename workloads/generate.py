"""Seeded tensor generators and page layout for the decode workloads.

Everything here is input preparation: random draws, rounding to the storage
type, page-pool layout, per-token fp8 scaling of the *inputs*, and overwriting
caller-chosen slots with NaN.  Which positions attention keeps, and every step
of attention itself, live elsewhere (the HIP library and, separately, the CPU
oracle); callers that need a retained mask build it themselves.
"""
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

from .configs import Config, QK_DIM, PAGE

FP8_MAX = 448.0  # largest finite OCP e4m3 value


@dataclass
class Inputs:
    q: torch.Tensor                 # bf16 [B, H, 576]
    kv_cache: torch.Tensor          # bf16 | float8_e4m3fn [num_pages, 128, 576]
    kv_scales: Optional[torch.Tensor]  # fp32 [num_pages, 128] (fp8 only)
    page_table: torch.Tensor        # int32 [B, max_pages]
    seq_lens: torch.Tensor          # int32 [B]  (host copy in seq_lens_host)
    seq_lens_host: list
    sink: int
    window: int
    softmax_scale: float
    kv_dtype: str

    @property
    def batch(self):
        return self.q.shape[0]

    @property
    def heads(self):
        return self.q.shape[1]

    @property
    def num_pages(self):
        return self.kv_cache.shape[0]

    @property
    def max_pages(self):
        return self.page_table.shape[1]


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def quantize_fp8_per_token(x: torch.Tensor):
    """x fp32 [..., 576] -> (float8_e4m3fn codes, fp32 scale [...]).

    scale = amax(|row|)/448 (1.0 for an all-zero row); code = round-to-nearest-
    even of x/scale, clamped to the finite range.  This prepares inputs only;
    how a code and its scale are turned back into a number is the decoder's
    business on each side.
    """
    amax = x.abs().amax(dim=-1)
    scale = torch.where(amax > 0, amax / FP8_MAX, torch.ones_like(amax))
    y = (x / scale.unsqueeze(-1)).clamp_(-FP8_MAX, FP8_MAX)
    return y.to(torch.float8_e4m3fn), scale.to(torch.float32)


def _fill_cache(num_pages, kv_dtype, kv_std, device, gen, chunk_pages=2048):
    if kv_dtype == "bf16":
        cache = torch.empty((num_pages, PAGE, QK_DIM), dtype=torch.bfloat16, device=device)
        scales = None
    elif kv_dtype == "fp8":
        cache = torch.empty((num_pages, PAGE, QK_DIM), dtype=torch.float8_e4m3fn, device=device)
        scales = torch.empty((num_pages, PAGE), dtype=torch.float32, device=device)
    else:
        raise ValueError(kv_dtype)
    for p0 in range(0, num_pages, chunk_pages):
        p1 = min(num_pages, p0 + chunk_pages)
        x = torch.randn((p1 - p0, PAGE, QK_DIM), dtype=torch.float32, device=device,
                        generator=gen) * kv_std
        if kv_dtype == "bf16":
            cache[p0:p1] = x.to(torch.bfloat16)
        else:
            c, s = quantize_fp8_per_token(x)
            cache[p0:p1] = c
            scales[p0:p1] = s
    return cache, scales


def make_custom(batch: int, heads: int, seq_lens: Sequence[int], sink: int, window: int,
                *, kv_dtype: str = "bf16", shuffled_pages: bool = True, seed: int = 0,
                q_std: float = 1.0 / 24.0, kv_std: float = 1.0 / 24.0,
                softmax_scale: float = 192.0 ** -0.5, spare_pages: int = 0,
                max_pages: Optional[int] = None, device="cpu") -> Inputs:
    """Build one decode problem.

    Sequence b owns ceil(L_b/128) physical pages.  With `shuffled_pages` the
    pool order is a seeded random permutation (plus `spare_pages` pages that no
    sequence references); otherwise pages are laid out sequence after sequence.
    Page-table entries past a sequence's last page are -1.
    """
    seq_lens = [int(x) for x in seq_lens]
    assert len(seq_lens) == batch
    device = torch.device(device)
    g = _gen(device, seed)
    pages_per_seq = [(L + PAGE - 1) // PAGE for L in seq_lens]
    used = sum(pages_per_seq)
    num_pages = max(1, used + spare_pages)
    mp = max(1, max(pages_per_seq) if pages_per_seq else 1)
    if max_pages is not None:
        assert max_pages >= mp
        mp = max_pages

    q = (torch.randn((batch, heads, QK_DIM), dtype=torch.float32, device=device, generator=g)
         * q_std).to(torch.bfloat16)
    cache, scales = _fill_cache(num_pages, kv_dtype, kv_std, device, g)

    if shuffled_pages:
        perm = torch.randperm(num_pages, device=device, generator=g)
    else:
        perm = torch.arange(num_pages, device=device)
    perm = perm.to(torch.int32).cpu()
    table = torch.full((batch, mp), -1, dtype=torch.int32)
    off = 0
    for b, n in enumerate(pages_per_seq):
        table[b, :n] = perm[off:off + n]
        off += n
    return Inputs(q=q, kv_cache=cache, kv_scales=scales,
                  page_table=table.to(device),
                  seq_lens=torch.tensor(seq_lens, dtype=torch.int32, device=device),
                  seq_lens_host=seq_lens, sink=int(sink), window=int(window),
                  softmax_scale=float(softmax_scale), kv_dtype=kv_dtype)


def make_planted(batch: int, heads: int, ctx: int, *, sink_tokens: int = 4, sink_logit: float = 6.0,
                 recency_logit: float = 6.0, recency_tau: float = 400.0, noise_std: float = 1.0,
                 seed: int = 0, device="cpu") -> Inputs:
    """A decode problem whose dense attention has the shape the paper's premise describes
    (section 3.2.1: the first tokens and the most recent tokens carry most of the attention
    mass): on top of Gaussian logits of standard deviation `noise_std`, position j gets
    `sink_logit` if j < sink_tokens and `recency_logit * exp(-(L-1-j)/recency_tau)`.

    The profile is planted through one coordinate: q[..., 575] = 1 and the cache row's last
    coordinate holds profile / softmax_scale; the other coordinates are random.  sink/window
    are left at "keep everything"; callers overwrite them.
    """
    scale = 192.0 ** -0.5
    # Gaussian part: logits = scale * sum_d q_d k_d over 575 coordinates with std noise_std
    std = (noise_std / (scale * (QK_DIM - 1) ** 0.5)) ** 0.5
    inp = make_custom(batch, heads, [ctx] * batch, 0, ctx, seed=seed, q_std=std, kv_std=std,
                      softmax_scale=scale, device=device)
    j = torch.arange(ctx, dtype=torch.float32)
    profile = recency_logit * torch.exp(-(ctx - 1 - j) / recency_tau)
    profile[:sink_tokens] += sink_logit
    col = (profile / scale).to(torch.bfloat16)
    inp.q[:, :, QK_DIM - 1] = 1.0
    for b in range(batch):
        for pg in range((ctx + PAGE - 1) // PAGE):
            n = min(PAGE, ctx - pg * PAGE)
            inp.kv_cache[int(inp.page_table[b, pg]), :n, QK_DIM - 1] = col[pg * PAGE: pg * PAGE + n].to(inp.kv_cache.device)
    return inp


def make_inputs(cfg: Config, device="cpu", *, batch: Optional[int] = None,
                seed_offset: int = 0) -> Inputs:
    """Inputs for one of the named workloads (optionally only its first
    `batch` sequences, for bounded CPU samples)."""
    B = cfg.batch if batch is None else int(batch)
    seed = cfg.seed + seed_offset
    if isinstance(cfg.ctx, tuple):
        lo, hi = cfg.ctx
        gl = torch.Generator(device="cpu")
        gl.manual_seed(seed + 7919)
        lens = torch.randint(lo, hi + 1, (cfg.batch,), generator=gl).tolist()[:B]
    else:
        lens = [int(cfg.ctx)] * B
    inp = make_custom(B, cfg.heads, lens, cfg.sink, cfg.window, kv_dtype=cfg.kv_dtype,
                      shuffled_pages=cfg.shuffled_pages, seed=seed, q_std=cfg.q_std,
                      kv_std=cfg.kv_std, softmax_scale=cfg.softmax_scale, device=device)
    if cfg.poison_tail:
        keep = [torch.arange(((L + PAGE - 1) // PAGE) * PAGE) < L for L in lens]
        poison_unretained(inp, keep, poison_unreferenced=False)
    return inp


def poison_unretained(inp: Inputs, keep, poison_unreferenced: bool = True) -> None:
    """Overwrite, in place, every cache slot the caller does not list as kept.

    keep[b][j] (j over the slots of sequence b's pages, in logical order) says
    which logical positions hold live data.  All other slots of referenced
    pages, and (optionally) all pages no sequence references, get NaN (bf16)
    or the e4m3 NaN code 0x7F with a NaN scale (fp8).
    """
    table = inp.page_table.cpu()
    dev = inp.kv_cache.device
    referenced = torch.zeros(inp.num_pages, dtype=torch.bool)
    slot_keep = torch.zeros((inp.num_pages, PAGE), dtype=torch.bool)
    for b, L in enumerate(inp.seq_lens_host):
        npg = (L + PAGE - 1) // PAGE
        kb = torch.as_tensor(keep[b], dtype=torch.bool)
        assert kb.numel() == npg * PAGE
        pages = table[b, :npg].long()
        referenced[pages] = True
        slot_keep[pages] = kb.view(npg, PAGE)
    dead = ~slot_keep
    if not poison_unreferenced:
        dead &= referenced.unsqueeze(1)
    dead = dead.to(dev)
    if inp.kv_dtype == "bf16":
        inp.kv_cache[dead] = float("nan")
    else:
        raw = inp.kv_cache.view(torch.uint8)
        raw[dead] = 0x7F
        inp.kv_scales[dead] = float("nan")
