"""Pins of the controller / planner oracle (oracle/planner.py) against what the paper and the mathematics fix:
the closed forms the paper prints (Section 3.2, Appendix B, the appendix on S_2), simulation of the cycle it
describes, special cases, and the hybrid-optimality theorem of Section 3.3."""
import math

import numpy as np
import pytest

import importlib.util
import os

if os.environ.get("LA_ORACLE_PLANNER_SRC"):      # the mutation test points this at a deliberately broken copy
    _spec = importlib.util.spec_from_file_location("planner_under_test", os.environ["LA_ORACLE_PLANNER_SRC"])
    P = importlib.util.module_from_spec(_spec)
    _spec.loader.exec_module(P)
else:
    from oracle import planner as P

GRID = [(a, c, k) for a in (0.3, 0.52, 0.66, 0.8, 0.93) for c in (0.05, 0.2, 0.3, 0.45) for k in (1, 2, 3, 4, 5, 8, 16)]


# ---- closed forms as printed ---------------------------------------------------------------------------------

def paper_f_sync(a, c, k):            # Section 3.2, sync speedup
    return (1 - a ** k) / ((1 - a) * (1 - c + c * k))


def paper_s1(a, c):                   # Section 3.2, case 1
    return 1 / (c + (1 - c) * (1 - a))


def paper_s2(a, c, k):                # Section 3.2, case 2
    return (1 - a ** k) / ((1 - a) + c * (a - a ** (k + 1) - k * (1 - a) * a ** k))


@pytest.mark.parametrize("a,c,k", GRID)
def test_sync_speedup_equals_the_printed_closed_form(a, c, k):
    assert P.speedup_sync(a, c, k) == pytest.approx(paper_f_sync(a, c, k), rel=1e-12)


@pytest.mark.parametrize("a,c,k", GRID)
def test_async_speedup_equals_the_printed_cases(a, c, k):
    want = paper_s1(a, c) if k >= math.ceil(1 / c) else paper_s2(a, c, k)
    assert P.speedup_async(a, c, k) == pytest.approx(want, rel=1e-12)


@pytest.mark.parametrize("a", [0.2, 0.52, 0.8, 0.95])
@pytest.mark.parametrize("k", [1, 2, 5, 9])
def test_expectations_of_the_s2_appendix(a, k):
    """E[X] = a/(1-a);  E ceil((X+1)/k) = 1/(1-a^k);  E[X mod k] = (a - a^(k+1) - k(1-a)a^k) / ((1-a)(1-a^k))."""
    assert P._expect(a, lambda x: x) == pytest.approx(a / (1 - a), rel=1e-13)
    assert P._expect(a, lambda x: -(-(x + 1) // k)) == pytest.approx(1 / (1 - a ** k), rel=1e-13)
    want = (a - a ** (k + 1) - k * (1 - a) * a ** k) / ((1 - a) * (1 - a ** k))
    assert P._expect(a, lambda x: x % k) == pytest.approx(want, rel=1e-12, abs=1e-13)   # the printed form cancels to ~1e-15 where the value is 0


# ---- the process itself, simulated ---------------------------------------------------------------------------

@pytest.mark.parametrize("a,c,k", [(0.6, 0.2, 4), (0.8, 0.1, 8), (0.52, 0.3, 2), (0.7, 0.25, 6)])
def test_sync_cycle_simulation(a, c, k):
    """Cycle by cycle: k-1 drafts one after the other (c each), one parallel target pass (1), drafts accepted
    independently with probability a until the first rejection; the target's step at the first rejection (or the
    bonus step) is emitted as well."""
    rng = np.random.default_rng(1)
    n = 400000
    accept = rng.random((n, k - 1)) < a
    accepted = np.where(accept.all(axis=1), k - 1, np.argmin(accept, axis=1)) if k > 1 else np.zeros(n, dtype=int)
    emitted = accepted + 1
    cost = (k - 1) * c + 1
    sim = emitted.mean() / cost
    err = 4 * emitted.std() / math.sqrt(n) / cost
    assert abs(sim - P.speedup_sync(a, c, k)) < err


@pytest.mark.parametrize("a,c,k", [(0.6, 0.2, 3), (0.8, 0.1, 8), (0.52, 0.3, 2), (0.7, 0.25, 6), (0.75, 0.3, 12)])
def test_async_stage_simulation(a, c, k):
    """Appendix B's stage model, sampled: X consecutive acceptances; the stage lasts 1 + cX when the draft is the
    slower side (k >= ceil(1/c)), else ceil((X+1)/k) + c (X mod k); it emits 1 + X steps."""
    rng = np.random.default_rng(2)
    n = 1000000
    x = rng.geometric(1 - a, size=n) - 1
    cost = 1 + c * x if k >= math.ceil(1 / c) else np.ceil((x + 1) / k) + c * (x % k)
    sim = (1 + x).sum() / cost.sum()
    # delta method for a ratio of means
    r = sim
    resid = (1 + x) - r * cost
    err = 4 * resid.std() / math.sqrt(n) / cost.mean()
    assert abs(sim - P.speedup_async(a, c, k)) < err


# ---- special cases -------------------------------------------------------------------------------------------

@pytest.mark.parametrize("a", [0.1, 0.6, 0.9])
@pytest.mark.parametrize("c", [0.05, 0.3])
def test_no_speculation_is_no_speedup(a, c):
    assert P.speedup_sync(a, c, 1) == pytest.approx(1.0, rel=1e-14)
    if math.ceil(1 / c) > 1:
        assert P.speedup_async(a, c, 1) == pytest.approx(1.0, rel=1e-13)


def test_limits():
    # a free draft: the speedup is the expected number of steps per cycle
    assert P.speedup_sync(0.7, 1e-12, 5) == pytest.approx(sum(0.7 ** i for i in range(5)), rel=1e-9)
    # a draft that is never accepted only costs time
    assert P.speedup_sync(1e-12, 0.2, 4) == pytest.approx(1 / (1 + 3 * 0.2), rel=1e-9)
    # deeper lookahead never hurts the async form below the depth limit, and it saturates at S_1-like values
    vals = [P.speedup_async(0.8, 0.1, k) for k in range(1, 10)]
    assert all(b > a for a, b in zip(vals, vals[1:]))
    # the speedup grows with the acceptance rate
    assert P.speedup_sync(0.8, 0.2, 4) > P.speedup_sync(0.6, 0.2, 4) > P.speedup_sync(0.4, 0.2, 4)


def test_parallel_dimension():
    assert P.parallel_dim_f(0.25, 3, True) == 3
    assert P.parallel_dim_f(0.25, 9, True) == 4          # min(ceil(1/c), k1)
    assert P.parallel_dim_f(0.3, 9, True) == 4
    assert P.parallel_dim_f(0.25, 9, False) == 9


# ---- Algorithm 1: verification and output construction ---------------------------------------------------------

def test_first_rejection():
    assert P.first_rejection([True, True, False, True]) == 2
    assert P.first_rejection([False, True, True]) == 0
    assert P.first_rejection([True, True, True]) == 3      # nothing rejected: the bonus step of the target
    assert P.first_rejection([]) == 0


def test_output_construction_follows_the_accepted_prefix():
    # three drafts of 5, 7 and 4 tokens; branch j sees drafts 0..j-1; the target's steps have 6, 3, 9, 2 tokens
    vis = [[0, 5, 12, 16]]
    own = [[6, 3, 9, 2]]
    assert P.output_construction([[True, False, True]], vis, own) == [(1, 1, 5, 3)]
    assert P.output_construction([[True, True, True]], vis, own) == [(3, 3, 16, 2)]
    assert P.output_construction([[False, True, True]], vis, own) == [(0, 0, 0, 6)]


# ---- Section 3.1, multi-branch drafting: the walk over a draft tree ---------------------------------------------

def full_tree(width, depth):
    """Parents of a tree with ``width`` alternatives per position, stored level by level."""
    par, level = [], [-1]
    for _ in range(depth):
        nxt = []
        for p in level:
            for _ in range(width):
                nxt.append(len(par))
                par.append(p)
        level = nxt
    return par


def test_tree_walk_worked_example():
    # position 0: drafts 0, 1;  below 0: drafts 2, 3;  below 1: drafts 4, 5.  own[j] = tokens of the target's step
    # that continues the bare prefix (j = 0) or the path ending in node j - 1
    par, own = [-1, -1, 0, 0, 1, 1], [[10, 11, 12, 13, 14, 15, 16]]
    walk = lambda v: P.tree_output_construction(par, [v], own)[0]
    assert walk([0, 0, 1, 1, 1, 1]) == (0, 0, 0, 10)                      # nothing at position 0 matched
    assert walk([0, 1, 1, 1, 0, 0]) == (1, 2, 0b000010, 12)               # node 1, none of its children (4, 5)
    assert walk([0, 1, 1, 1, 0, 1]) == (2, 6, 0b100010, 16)               # node 1 then node 5
    assert walk([1, 1, 0, 1, 1, 1]) == (2, 4, 0b001001, 14)               # 0 and 1 both match: 0; then 3
    assert walk([1, 0, 1, 1, 0, 0]) == (2, 3, 0b000101, 13)               # 2 and 3 both match: 2


def test_a_tree_of_width_one_is_algorithm_1s_chain():
    rng = np.random.default_rng(11)
    for drafts in (0, 1, 4, 9):
        par = list(range(-1, drafts - 1))
        v = (rng.random((50, drafts)) < 0.7).tolist()
        own = rng.integers(1, 30, size=(50, drafts + 1)).tolist()
        vis = [list(range(drafts + 1))] * 50                          # one token per draft: vis = number accepted
        chain = P.output_construction(v, vis, own)
        tree = P.tree_output_construction(par, v, own)
        for (j, src, nch, nown), (d, tsrc, mask, town) in zip(chain, tree):
            assert (d, tsrc, town) == (j, src, nown)
            assert mask == (1 << j) - 1 and nch == j


@pytest.mark.parametrize("width,depth", [(2, 2), (3, 2), (2, 3)])
def test_tree_walk_is_the_unique_greedy_path(width, depth):
    """Stated without the walk: the accepted set is a path from the top (every member's parent is the previous
    member), each member matched and no earlier sibling did, and nothing below the last member matched."""
    par = full_tree(width, depth)
    n = len(par)
    rng = np.random.default_rng(width * 10 + depth)
    for _ in range(300):
        v = (rng.random(n) < 0.5).tolist()
        d, src, mask, own = P.tree_output_construction(par, [v], [list(range(100, 101 + n))])[0]
        members = [i for i in range(n) if mask >> i & 1]
        assert len(members) == d and own == 100 + src
        prev = -1
        for m in members:
            assert par[m] == prev and v[m]
            assert not any(v[s] for s in range(m) if par[s] == prev)
            prev = m
        assert src == prev + 1
        assert not any(v[c] for c in range(n) if par[c] == prev)


@pytest.mark.parametrize("width,depth", [(1, 3), (2, 2), (3, 2), (2, 3)])
def test_accepted_depth_under_independent_verdicts(width, depth):
    """Every draft matching independently with probability a: a position succeeds when any of its ``width``
    alternatives matches, so P(depth >= d) = (1 - (1 - a)^width)^d (the reason for drafting several alternatives).
    Checked by summing over all verdict patterns."""
    par = full_tree(width, depth)
    n, a = len(par), 0.37
    reach = [0.0] * (depth + 1)
    for pattern in range(1 << n):
        v = [(pattern >> i) & 1 for i in range(n)]
        w = np.prod([a if x else 1 - a for x in v])
        d = P.tree_output_construction(par, [v], [[1] * (n + 1)])[0][0]
        for k in range(d + 1):
            reach[k] += w
    for d in range(depth + 1):
        assert reach[d] == pytest.approx((1 - (1 - a) ** width) ** d, rel=1e-12)


# ---- Section 3.3 -----------------------------------------------------------------------------------------------

def test_plan_respects_the_budget_and_is_the_maximum():
    for asyn in (False, True):
        k1, k2, h, table = P.plan(0.7, 0.2, 0.65, 0.1, 16, asyn)
        assert P.parallel_dim_f(0.2, k1, asyn) * k2 <= 16
        assert h == max(table.values())
        assert all(P.parallel_dim_f(0.2, a, asyn) * b <= 16 for a, b in table)
        # pure strategies are in the table
        assert (1, 16) in table and (16 if not asyn else 5, 1) in table


def test_combined_speedup_is_the_product_of_the_printed_forms():
    """h(k1, k2) = f(k1) g(k2) (Section 3.3) with f from (alpha_1, c_1) and g from (alpha_2, c_2)."""
    a1, c1, a2, c2 = 0.7, 0.2, 0.55, 0.08
    _, _, _, table = P.plan(a1, c1, a2, c2, 12, False)
    for (k1, k2), h in table.items():
        assert h == pytest.approx(paper_f_sync(a1, c1, k1) * paper_f_sync(a2, c2, k2), rel=1e-12)
    _, _, _, table = P.plan(a1, c1, a2, c2, 12, True)
    for (k1, k2), h in table.items():
        f = paper_s1(a1, c1) if k1 >= 5 else paper_s2(a1, c1, k1)
        assert h == pytest.approx(f * paper_f_sync(a2, c2, k2), rel=1e-12)
    assert P.combined(a1, c1, 3, a2, c2, 4, True) == pytest.approx(table[(3, 4)], rel=1e-14)


@pytest.mark.parametrize("a1", [0.53, 0.6, 0.7, 0.79])
@pytest.mark.parametrize("a2", [0.53, 0.66, 0.79])
@pytest.mark.parametrize("c1", [0.1, 0.2, 0.33])
@pytest.mark.parametrize("c2", [0.05, 0.19])
@pytest.mark.parametrize("M", [16, 24, 32])
def test_hybrid_optimality_theorem(a1, a2, c1, c2, M):
    """Section 3.3, theorem for the async algorithm: for 0.52 < a1, a2 < 0.8, c1 < 1/3, c2 < 1/5 and M >= 16 the
    maximum is attained only by hybrid strategies (k1 >= 2 and k2 >= 2)."""
    k1, k2, h, table = P.plan(a1, c1, a2, c2, M, True)
    assert k1 >= 2 and k2 >= 2
    best_pure = max(v for (x, y), v in table.items() if x == 1 or y == 1)
    assert h > best_pure
