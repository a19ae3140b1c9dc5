"""CPU oracle of the step-level controller and the budget planner.  TEST INFRASTRUCTURE ONLY (see ``la_oracle.c``):
nothing in the product package imports this module, and it shares no code with the library's host functions.

Everything is written from the *process* the paper describes, not from its closed forms, so that the closed forms
(which the library evaluates) are checked against something else:

* Algorithm 1, verification and output construction: ``j*`` is the first draft step the verifier rejects (or the
  number of drafts when none is), the output is the accepted drafts followed by the target's step ``j*``.
* Section 3.1, "Multi-Branch Drafting": several alternative drafts per position; the target's step for a position is
  checked against every alternative drafted behind the accepted path, one that matches is kept and the walk goes on
  below it, the others are discarded.  Which of several matching alternatives is kept the paper does not say: the
  one drafted first (smallest node number).
* Section 3.2 / Appendix B, step-level speedups.  ``X`` = number of consecutively accepted drafts,
  ``P(X = n) = alpha^n (1 - alpha)``.
    - sync, ``k`` target steps in parallel (so ``k - 1`` drafts, generated one after the other): a cycle costs
      ``(k - 1) c + 1`` target-step times and emits ``min(X, k - 1) + 1`` steps;
    - async, draft slower than the depth limit (``k >= ceil(1/c)``): a stage costs ``1 + c X`` and emits ``1 + X``;
    - async, depth limited (``k < ceil(1/c)``): a stage costs ``ceil((X + 1)/k) + c (X mod k)`` and emits ``1 + X``.
  The speedup is expected emitted steps over expected cost (law of large numbers over stages).  Expectations are
  plain sums over the geometric law, carried until the tail is below 1e-18 of the running value.
* Section 3.3: token-level speculation inside a step has the sync form with ``(alpha_2, c_2, k_2)``; the combined
  speedup is the product; the plan is the argmax over integers ``k_1, k_2 >= 1`` with
  ``ParallelDim_f * k_2 <= M``, ``ParallelDim_f = k_1`` (sync) or ``min(ceil(1/c_1), k_1)`` (async), found by
  trying every pair.  Ties (the paper does not say): smallest ``k_1``, then smallest ``k_2``.
"""
from __future__ import annotations

import math
from typing import Callable, List, Sequence, Tuple


def first_rejection(verdicts: Sequence[bool]) -> int:
    """Algorithm 1: j* = min({j : V(s_j, s^_j) is False} U {number of drafts})."""
    for j, ok in enumerate(verdicts):
        if not ok:
            return j
    return len(verdicts)


def output_construction(verdicts: Sequence[Sequence[bool]], chain_vis: Sequence[Sequence[int]],
                        own_len: Sequence[Sequence[int]]) -> List[Tuple[int, int, int, int]]:
    """Per request: (j*, surviving branch, chain tokens kept, own tokens kept).  Branch j verifies position j; it sees
    ``chain_vis[j]`` tokens of the drafted chain (the drafts 0..j-1) and holds ``own_len[j]`` tokens of the target's
    step j.  The output (accepted drafts, then the target's step j*) is what branch j* saw plus what it produced."""
    out = []
    for v, vis, own in zip(verdicts, chain_vis, own_len):
        j = first_rejection(v)
        out.append((j, j, int(vis[j]), int(own[j])))
    return out


def tree_output_construction(parent: Sequence[int], verdicts: Sequence[Sequence[bool]],
                             own_len: Sequence[Sequence[int]]) -> List[Tuple[int, int, int, int]]:
    """Draft tree: node n hangs below node ``parent[n]`` (-1 = directly below the accepted text).  Branch 0 is the
    target's step after the bare prefix, branch 1 + n its step after the path ending in node n; ``verdicts[b][n]``
    says whether draft n matched the target's step of branch ``1 + parent[n]``.  Per request:
    (accepted depth, surviving branch, bit set of the accepted nodes, own tokens kept)."""
    out = []
    for v, own in zip(verdicts, own_len):
        here, accepted = -1, []
        while True:
            alternatives = [n for n in range(len(parent)) if parent[n] == here]
            matching = [n for n in alternatives if v[n]]
            if not matching:
                break
            here = min(matching)
            accepted.append(here)
        out.append((len(accepted), here + 1, sum(1 << n for n in accepted), int(own[here + 1])))
    return out


def _expect(alpha: float, fn: Callable[[int], float]) -> float:
    """E[fn(X)] for P(X = n) = alpha^n (1 - alpha): direct summation."""
    total, n, w = 0.0, 0, 1.0 - alpha
    while True:
        total += w * fn(n)
        n += 1
        w *= alpha
        # what is left is at most  alpha^n * sup|fn| ; fn grows at most linearly here
        if w * (n + 1) / (1.0 - alpha) ** 2 < 1e-18 * max(1.0, abs(total)):
            return total


def speedup_sync(alpha: float, c: float, k: int) -> float:
    emitted = _expect(alpha, lambda x: min(x, k - 1) + 1)
    return emitted / ((k - 1) * c + 1.0)


def depth_limit(c: float) -> int:
    return int(math.ceil(1.0 / c))


def speedup_async(alpha: float, c: float, k: int) -> float:
    emitted = _expect(alpha, lambda x: 1 + x)
    if k >= depth_limit(c):
        cost = _expect(alpha, lambda x: 1 + c * x)
    else:
        cost = _expect(alpha, lambda x: -(-(x + 1) // k) + c * (x % k))
    return emitted / cost


def parallel_dim_f(c1: float, k1: int, asynchronous: bool) -> int:
    return min(depth_limit(c1), k1) if asynchronous else k1


def combined(alpha1, c1, k1, alpha2, c2, k2, asynchronous: bool) -> float:
    f = speedup_async(alpha1, c1, k1) if asynchronous else speedup_sync(alpha1, c1, k1)
    return f * speedup_sync(alpha2, c2, k2)


def plan(alpha1, c1, alpha2, c2, budget: int, asynchronous: bool):
    """Every pair tried.  Returns (k1, k2, h, table) with table[(k1, k2)] = h for all feasible pairs."""
    f = {k1: (speedup_async(alpha1, c1, k1) if asynchronous else speedup_sync(alpha1, c1, k1))
         for k1 in range(1, budget + 1)}
    g = {k2: speedup_sync(alpha2, c2, k2) for k2 in range(1, budget + 1)}
    table = {}
    best = None
    for k1 in range(1, budget + 1):
        for k2 in range(1, budget + 1):
            if parallel_dim_f(c1, k1, asynchronous) * k2 > budget:
                continue
            h = f[k1] * g[k2]
            table[(k1, k2)] = h
            if best is None or h > best[2]:
                best = (k1, k2, h)
    return best[0], best[1], best[2], table
