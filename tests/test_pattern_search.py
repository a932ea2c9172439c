"""Layer-pattern search (paper section 3.2.2): the genetic search against exhaustive search on
small layer counts (CPU), and the per-pattern latency on the GPU with one captured graph per
pattern, replayed several times and compared with eager results."""
import dataclasses
import itertools

import pytest
import torch

from paper_2511_22481_amd.pattern_search import LayerStack, additive_accuracy, evolve, search


@pytest.mark.parametrize("n,seed,tau", [(8, 1, 0.8), (10, 2, 0.9), (12, 3, 0.7), (10, 4, 0.999), (6, 5, 0.2)])
def test_search_matches_exhaustive_optimum(n, seed, tau):
    acc = additive_accuracy(n, seed=seed)
    # exhaustive: the largest number of compressed layers that still reaches tau (latency falls
    # with every compressed layer)
    best_k = max((sum(p) for p in itertools.product((0, 1), repeat=n) if acc(p) >= tau), default=None)
    got = search(acc, n, tau, latency=lambda k: 10.0 * (n - k) + 1.0 * k, seed=seed)
    assert best_k is not None and got is not None
    assert got["accuracy"] >= tau and sum(got["pattern"]) == got["compressed_layers"] == best_k
    assert got["latency"] == 10.0 * (n - best_k) + best_k


def test_evolve_keeps_the_layer_count_and_improves():
    n, k = 24, 9
    acc = additive_accuracy(n, seed=7)
    first, a0, _ = evolve(acc, n, k, tau=2.0, generations=0, seed=1)
    best, a1, gens = evolve(acc, n, k, tau=2.0, generations=60, seed=1)
    assert sum(first) == sum(best) == k and a1 >= a0
    optimum = 1.0 - sum(sorted(acc.sensitivities)[:k])
    assert a1 >= optimum - 0.02          # close to compressing the k least sensitive layers
    assert search(acc, n, tau=1.5) is None


@pytest.mark.gpu
def test_one_graph_per_pattern_replays_like_eager():
    import parity
    from workloads import make_custom
    lens = [700, 64, 2500]
    layers = [parity.to_device(make_custom(3, 32, lens, 0, 4096, seed=60 + l, q_std=0.5, kv_std=0.5))
              for l in range(4)]
    stack = LayerStack(layers, sink=32, window=200)
    for pattern in [(0, 0, 0, 0), (1, 0, 1, 1), (1, 1, 1, 1)]:
        g = stack.graph(pattern)
        for _ in range(3):                       # replays with eager work and syncs in between
            stack.out.zero_()
            g.replay()
            torch.cuda.synchronize()
            got, got_lse = stack.out.clone(), stack.lse.clone()
            stack.out.zero_()
            stack.step(pattern)
            torch.cuda.synchronize()
            assert torch.equal(got, stack.out) and torch.equal(got_lse, stack.lse)
        # the last layer's result is what the buffers hold: check it against the oracle
        sw = (32, 200) if pattern[-1] else (0, max(lens))
        last = dataclasses.replace(layers[-1], sink=sw[0], window=sw[1])
        parity.assert_parity(last, stack.out, stack.lse, row_rel_l2=1e-2, what=f"pattern {pattern}")
    t_dense, t_comp = stack.time((0, 0, 0, 0)), stack.time((1, 1, 1, 1))
    assert t_comp < t_dense


def test_search_at_the_models_depth():
    """61 layers (DeepSeek-R1's depth).  For the stand-in accuracy the optimum is known (compress
    the least sensitive layers: 35 of 61 here).  The genetic search is a heuristic: with its
    default budget it stops at 29 layers, with population 64 and 200 generations at 34; it never
    returns a pattern below the accuracy floor or above the optimum."""
    n = 61
    acc = additive_accuracy(n, seed=3)
    sens = sorted(acc.sensitivities)
    tau = 0.9
    k_opt = max(k for k in range(n + 1) if 1.0 - sum(sens[:k]) >= tau)
    for kw, slack in ((dict(), 7), (dict(generations=200, population=64), 2)):
        res = search(acc, n, tau, seed=5, **kw)
        assert res is not None and len(res["pattern"]) == n
        assert res["accuracy"] >= tau and res["compressed_layers"] == sum(res["pattern"])
        assert k_opt - slack <= res["compressed_layers"] <= k_opt, (kw, res["compressed_layers"], k_opt)


@pytest.mark.gpu
def test_layer_stack_at_the_models_depth():
    """Latency(p) over 61 layers, one captured graph per pattern: compressing more layers must
    not make the step slower, replay equals eager bitwise, the last layer matches the oracle."""
    import parity
    from workloads import make_custom
    n, lens = 61, [3000, 900, 4000, 2200]
    layers = [parity.to_device(make_custom(len(lens), 64, lens, 0, 4096, seed=200 + l, q_std=0.5, kv_std=0.5))
              for l in range(n)]
    stack = LayerStack(layers, sink=64, window=512)
    times = {}
    for k in (0, 15, 30, 45, 61):
        pattern = tuple([1] * k + [0] * (n - k))
        times[k] = stack.time(pattern, reps=5)
    print("latency ms by compressed layers:", times)
    assert times[61] < times[30] < times[0]
    pattern = tuple(int((l * 7) % 3 == 0) for l in range(n))
    g = stack.graph(pattern)
    for _ in range(2):
        stack.out.zero_()
        g.replay()
        torch.cuda.synchronize()
        got, got_lse = stack.out.clone(), stack.lse.clone()
        stack.out.zero_()
        stack.step(pattern)
        torch.cuda.synchronize()
        assert torch.equal(got, stack.out) and torch.equal(got_lse, stack.lse)
    sw = (64, 512) if pattern[-1] else (0, max(lens))
    last = dataclasses.replace(layers[-1], sink=sw[0], window=sw[1])
    parity.assert_parity(last, stack.out, stack.lse, row_rel_l2=1e-2, what="61 layers")
