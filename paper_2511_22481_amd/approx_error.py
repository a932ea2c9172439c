"""How far the kept-set attention is from dense attention (paper section 3.2.1, first
equation: the "approximately equal" between attention over all keys and attention over the
sink + recent keys), on synthetic inputs whose dense attention has planted sink and recency
mass.  Both sides are computed by the decode library; dense = every position kept.

    python -m paper_2511_22481_amd.approx_error [--ctx 8192] [--batch 4] [--heads 128]

Prints one line per (S, W): relative L2 distance of the outputs and the largest lse gap.
"""
import argparse
import json


def sweep(inp, settings):
    """inp: a decode problem on the GPU (workloads.Inputs).  Returns a list of dicts."""
    import torch
    from . import decode
    L = max(inp.seq_lens_host)
    dense, dense_lse, _ = decode(inp.q, inp.kv_cache, inp.kv_scales, inp.page_table,
                                 inp.seq_lens_host, 0, L, inp.softmax_scale, out_dtype=torch.float32)
    rows = []
    for S, W in settings:
        out, lse, plan = decode(inp.q, inp.kv_cache, inp.kv_scales, inp.page_table,
                                inp.seq_lens_host, S, W, inp.softmax_scale, out_dtype=torch.float32)
        torch.cuda.synchronize()
        rel = float((out - dense).norm() / dense.norm())
        # lse gap = -log of the softmax mass the kept set holds
        gap = float((dense_lse - lse).max())
        rows.append({"sink": S, "window": W, "kept_fraction": plan.retained_tokens / (L * len(inp.seq_lens_host)),
                     "rel_l2_vs_dense": rel, "max_lse_gap": gap, "min_kept_mass": float(torch.exp(-(dense_lse - lse)).min())})
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--ctx", type=int, default=8192)
    ap.add_argument("--batch", type=int, default=4)
    ap.add_argument("--heads", type=int, default=128)
    args = ap.parse_args()
    import torch
    from workloads import make_planted
    if not torch.cuda.is_available():
        raise SystemExit("needs a GPU: the decode library has no CPU path")
    inp = make_planted(args.batch, args.heads, args.ctx, seed=11, device="cuda:0")
    settings = [(0, 128), (4, 128), (4, 512), (128, 512), (128, 2048), (128, 4096), (128, args.ctx)]
    for r in sweep(inp, settings):
        print(json.dumps(r))


if __name__ == "__main__":
    main()
