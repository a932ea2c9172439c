"""Layer-wise compression patterns (paper section 3.2.2).

A pattern p in {0,1}^n says which of a model's n attention layers keep only the sink + recent
tokens (p_l = 1) and which stay dense (p_l = 0).  The paper searches, with a genetic algorithm
and the model's accuracy on held-out data as fitness, for

        min_p Latency(p)   subject to   Acc(p) >= tau.

What this module provides
  * `search`: that genetic search (random initial population; selection, crossover and mutation
    over generations; early stop once a pattern reaches tau), for any accuracy function the caller
    supplies.  With identical layers the latency depends only on how many layers are compressed,
    so the search walks that number down from n and, for each, evolves patterns with exactly that
    many compressed layers towards higher accuracy; the first count for which tau is reached is
    the minimum-latency answer.
  * `LayerStack`: the latency side on the GPU: one decode launch per layer on shared buffers (dense
    layers keep every position), captured into one graph per pattern and timed by replay.
The accuracy of a real model is outside this library; tests and the demo use a stand-in
(`additive_accuracy`: a seeded per-layer sensitivity, accuracy = 1 - sum of the compressed
layers' sensitivities), which says nothing about any trained model.
"""
import math
import random


def additive_accuracy(n_layers, seed=0, total_drop=0.5):
    """A stand-in for Acc(p): layer l costs sens[l] accuracy when compressed; the sensitivities
    are seeded, positive and sum to `total_drop`."""
    rng = random.Random(seed)
    raw = [rng.random() ** 3 + 0.02 for _ in range(n_layers)]
    tot = sum(raw)
    sens = [total_drop * r / tot for r in raw]

    def acc(p):
        return 1.0 - sum(s for s, bit in zip(sens, p) if bit)
    acc.sensitivities = sens
    return acc


def _random_pattern(rng, n, k):
    on = set(rng.sample(range(n), k))
    return tuple(1 if i in on else 0 for i in range(n))


def _repair(rng, p, k):
    """Bring a child back to exactly k compressed layers."""
    p = list(p)
    ones = [i for i, b in enumerate(p) if b]
    zeros = [i for i, b in enumerate(p) if not b]
    rng.shuffle(ones)
    rng.shuffle(zeros)
    while len(ones) > k:
        i = ones.pop()
        p[i] = 0
        zeros.append(i)
    while len(ones) < k:
        i = zeros.pop()
        p[i] = 1
        ones.append(i)
    return tuple(p)


def evolve(acc, n, k, tau, *, population=32, generations=40, mutation=0.05, seed=0):
    """Genetic search among patterns with exactly k compressed layers for high accuracy.
    Returns (best pattern, its accuracy, generations used); stops early at accuracy >= tau."""
    rng = random.Random(seed * 1000003 + k)
    population = min(population, math.comb(n, k))       # no more than the distinct patterns there are
    pop = list({_random_pattern(rng, n, k) for _ in range(population)})
    best, best_acc = None, -1.0
    for gen in range(generations + 1):
        scored = sorted(((acc(p), p) for p in pop), reverse=True)
        if scored[0][0] > best_acc:
            best_acc, best = scored[0]
        if best_acc >= tau or gen == generations:
            return best, best_acc, gen
        parents = [p for _, p in scored[:max(2, len(scored) // 2)]]       # selection
        children = {best}                                                  # elitism
        for _ in range(8 * population):                                    # bounded: children may repeat
            if len(children) >= population:
                break
            a, b = rng.sample(parents, 2) if len(parents) > 1 else (parents[0], parents[0])
            cut = rng.randrange(1, n) if n > 1 else 0                      # one-point crossover
            child = list(a[:cut] + b[cut:])
            for i in range(n):                                             # mutation
                if rng.random() < mutation:
                    child[i] ^= 1
            children.add(_repair(rng, child, k))
        pop = list(children)
    return best, best_acc, generations


def search(acc, n_layers, tau, latency=None, **ga):
    """min Latency(p) s.t. Acc(p) >= tau.  `latency(k)` (optional) gives the latency with k
    compressed layers for the report; it must not increase with k.  Returns a dict with the
    pattern, its accuracy, the number of compressed layers and (if given) the latency."""
    for k in range(n_layers, -1, -1):
        p, a, gens = evolve(acc, n_layers, k, tau, **ga)
        if a >= tau:
            return {"pattern": p, "accuracy": a, "compressed_layers": k, "generations": gens,
                    "latency": latency(k) if latency else None}
    return None  # even the uncompressed model misses tau


class LayerStack:
    """n attention layers over the same shapes: layer l decodes with (sink, window) if p_l = 1 and
    densely if p_l = 0.  Every layer has its own cache (as in a model); q/out buffers are shared.
    `graph(p)` captures one decode step over all layers; `time(p)` replays it."""

    def __init__(self, layer_inputs, sink, window):
        import torch
        from . import omniattn_plan, BF16, FP8_E4M3
        self.layers = layer_inputs
        i0 = layer_inputs[0]
        batch, heads = i0.q.shape[0], i0.q.shape[1]
        kw = dict(batch=batch, num_heads=heads, max_pages_per_seq=i0.page_table.shape[1],
                  num_pages=i0.kv_cache.shape[0], softmax_scale=i0.softmax_scale,
                  kv_dtype=FP8_E4M3 if i0.kv_dtype == "fp8" else BF16)
        L = max(i0.seq_lens_host)
        self.plans = {1: omniattn_plan(i0.seq_lens_host, sink=sink, window=window, **kw),
                      0: omniattn_plan(i0.seq_lens_host, sink=0, window=L, **kw)}
        dev = i0.q.device
        self.out = torch.empty((batch, heads, 512), dtype=torch.bfloat16, device=dev)
        self.lse = torch.empty((batch, heads), dtype=torch.float32, device=dev)
        ws = max(max(p.workspace_bytes for p in self.plans.values()), 256)
        self.ws = torch.empty(ws, dtype=torch.uint8, device=dev)

    def step(self, pattern, stream=None):
        from . import omniattn_decode
        for bit, inp in zip(pattern, self.layers):
            omniattn_decode(self.plans[int(bit)], inp.q, inp.kv_cache, inp.kv_scales, inp.page_table,
                            self.out, self.lse, self.ws, stream)

    def graph(self, pattern):
        import torch
        g = torch.cuda.CUDAGraph()
        self.step(pattern)                       # warm up outside the capture
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            self.step(pattern, torch.cuda.current_stream())
        return g

    def time(self, pattern, reps=20):
        """Milliseconds per decode step over all layers (graph replay)."""
        import torch
        g = self.graph(pattern)
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps


def main():
    """Demo on synthetic inputs: measure the step latency for every number of compressed layers
    (graph replay), then search with the stand-in accuracy."""
    import argparse
    import json
    import torch
    from workloads import make_custom
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=8)
    ap.add_argument("--batch", type=int, default=16)
    ap.add_argument("--heads", type=int, default=128)
    ap.add_argument("--seq-len", type=int, default=32768)
    ap.add_argument("--sink", type=int, default=128)
    ap.add_argument("--window", type=int, default=2048)
    ap.add_argument("--tau", type=float, default=0.9)
    a = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("pattern_search: needs a GPU (the latency term is measured, not modelled)")
    layers = [make_custom(a.batch, a.heads, [a.seq_len] * a.batch, a.sink, a.window, seed=l, device="cuda")
              for l in range(a.layers)]
    stack = LayerStack(layers, a.sink, a.window)
    lat = {k: stack.time(tuple([1] * k + [0] * (a.layers - k))) for k in range(a.layers + 1)}
    res = search(additive_accuracy(a.layers, seed=1), a.layers, a.tau, latency=lat.get)
    print(json.dumps({"latency_ms_by_compressed_layers": lat, "search": res}))


if __name__ == "__main__":
    main()
