"""Choice of the grouping configuration of one layer (Appendix B, Alg. 5).

Every (tolerance, threshold) pair of the search space runs the grouped matmul of Alg. 4
(``ts_grouped_matmul_adaptive``) on each sampled input; the pair with the smallest summed time wins.
The time is taken with HIP events on the library's stream unless a cost function is given
(host-only tests pass one).
"""
from __future__ import annotations

import itertools
from typing import Callable, Iterable, Sequence

DEFAULT_EPS_SPACE = (0.0, 0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.8, 1.0)
DEFAULT_S_SPACE = (0, 10_000, 30_000, 100_000, 1 << 40)


def measured_cost(iters: int = 10, warmup: int = 3) -> Callable:
    """Cost function for :func:`adaptive_group_search`: average microseconds of one grouped matmul.
    A sample is ``(F, feats_or_None, weights, kmap, G)`` of device tensors and a built map."""
    import torch
    from . import binding as ts

    def cost(sample, eps, S):
        F, feats, weights, kmap, G = sample
        for _ in range(warmup):
            ts.ts_grouped_matmul_adaptive(F, feats, weights, kmap, eps, S, G)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            ts.ts_grouped_matmul_adaptive(F, feats, weights, kmap, eps, S, G)
        b.record()
        b.synchronize()
        return a.elapsed_time(b) * 1e3 / iters

    return cost


def adaptive_group_search(samples: Iterable, eps_space: Sequence[float] = DEFAULT_EPS_SPACE,
                          S_space: Sequence[int] = DEFAULT_S_SPACE, cost: Callable | None = None):
    """Returns ``(eps, S, total_cost, table)``; ``table[(eps, S)]`` holds every pair's summed cost."""
    samples = list(samples)
    cost = cost or measured_cost()
    table = {pair: sum(cost(sample, *pair) for sample in samples) for pair in itertools.product(eps_space, S_space)}
    if not table:
        raise ValueError("empty search space")
    eps, S = min(table, key=table.get)      # the first pair in search order among equals
    return eps, S, table[(eps, S)], table
