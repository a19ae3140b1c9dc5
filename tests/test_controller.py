"""The library's host-only controller and planner against the oracle (oracle/planner.py).  No GPU involved: these
functions run on the CPU, so the parity tests do too.  Integers are compared exactly; the closed forms (fp64) must
agree with the oracle's summed expectations to 1e-12 relative."""
import numpy as np
import pytest

from oracle import planner as P
from paper_2506_19830_amd import binding as B

GRID = [(a, c, k) for a in (0.05, 0.3, 0.52, 0.66, 0.8, 0.93, 0.99) for c in (0.01, 0.05, 0.2, 0.3, 0.45, 0.9)
        for k in (1, 2, 3, 4, 5, 8, 16, 64)]


@pytest.mark.parametrize("a,c,k", GRID)
def test_speedup_forms_match_the_oracle(a, c, k):
    assert B.la_speedup_step_sync(a, c, k) == pytest.approx(P.speedup_sync(a, c, k), rel=1e-12)
    assert B.la_speedup_token(a, c, k) == pytest.approx(P.speedup_sync(a, c, k), rel=1e-12)
    assert B.la_speedup_step_async(a, c, k) == pytest.approx(P.speedup_async(a, c, k), rel=1e-12)


def test_step_select_matches_the_oracle_on_random_verdicts():
    rng = np.random.default_rng(3)
    for nb in (1, 2, 5, 9):
        nreq = 64
        verdicts = rng.random((nreq, nb - 1)) < 0.7
        vis = np.sort(rng.integers(0, 500, size=(nreq, nb)), axis=1)
        vis[:, 0] = 0
        own = rng.integers(1, 65, size=(nreq, nb))
        j, src, nch, nown = B.la_step_select(verdicts, vis, own)
        want = P.output_construction(verdicts.tolist(), vis.tolist(), own.tolist())
        assert [tuple(int(x) for x in t) for t in zip(j, src, nch, nown)] == want


def test_step_select_edge_cases():
    j, src, nch, nown = B.la_step_select([[True, True, True]], [[0, 5, 12, 16]], [[6, 3, 9, 2]])
    assert (j[0], src[0], nch[0], nown[0]) == (3, 3, 16, 2)
    j, src, nch, nown = B.la_step_select([[False, True, True]], [[0, 5, 12, 16]], [[6, 3, 9, 2]])
    assert (j[0], src[0], nch[0], nown[0]) == (0, 0, 0, 6)


def random_tree(rng, nodes):
    """Any tree with parents before children (not only the full ones the generators make)."""
    return [int(rng.integers(-1, n)) for n in range(nodes)]


def test_tree_select_matches_the_oracle_on_random_trees():
    rng = np.random.default_rng(4)
    for nodes in (0, 1, 2, 7, 30, 64):
        for accept in (0.3, 0.7, 0.95):
            par = random_tree(rng, nodes)
            nreq = 40
            verdicts = rng.random((nreq, nodes)) < accept
            own = rng.integers(1, 65, size=(nreq, nodes + 1))
            depth, mask, src, nown = B.la_step_select_tree(par, verdicts, own)
            want = P.tree_output_construction(par, verdicts.tolist(), own.tolist())
            assert [tuple(int(x) for x in t) for t in zip(depth, src, mask, nown)] == want


def test_tree_select_of_a_chain_is_step_select():
    rng = np.random.default_rng(5)
    drafts, nreq = 6, 50
    verdicts = rng.random((nreq, drafts)) < 0.8
    own = rng.integers(1, 20, size=(nreq, drafts + 1))
    vis = np.tile(np.arange(drafts + 1), (nreq, 1))
    j, src, nch, nown = B.la_step_select(verdicts, vis, own)
    depth, mask, tsrc, town = B.la_step_select_tree(np.arange(-1, drafts - 1), verdicts, own)
    assert np.array_equal(depth, j) and np.array_equal(tsrc, src) and np.array_equal(town, nown)
    assert np.array_equal(mask, (np.uint64(1) << j.astype(np.uint64)) - np.uint64(1))


def test_tree_select_uses_all_64_bits():
    par = list(range(-1, 63))                                      # a chain of 64 drafts, all accepted
    depth, mask, src, nown = B.la_step_select_tree(par, np.ones((1, 64), bool), np.arange(65)[None])
    assert depth[0] == 64 and mask[0] == np.uint64(2 ** 64 - 1) and src[0] == 64 and nown[0] == 64


def test_tree_select_rejects_malformed_trees():
    own = np.ones((1, 4), dtype=np.int32)
    v = np.ones((1, 3), dtype=bool)
    for par in ([-1, 1, 0], [-1, 0, 2], [-2, 0, 1], [0, 0, 1]):       # a node that is its own ancestor / child first
        with pytest.raises(B.LaError):
            B.la_step_select_tree(par, v, own)
    with pytest.raises(B.LaError):
        B.la_step_select_tree(list(range(-1, 64)), np.ones((1, 65), bool), np.ones((1, 66), np.int32))   # 65 nodes


PLAN_GRID = [(a1, c1, a2, c2, M, asyn) for a1 in (0.3, 0.6, 0.79, 0.95) for c1 in (0.04, 0.2, 0.33, 0.6)
             for a2 in (0.4, 0.7) for c2 in (0.05, 0.3) for M in (1, 4, 16, 33) for asyn in (False, True)]


@pytest.mark.parametrize("a1,c1,a2,c2,M,asyn", PLAN_GRID)
def test_plan_matches_exhaustive_search(a1, c1, a2, c2, M, asyn):
    k1, k2, h = B.la_plan_budget(a1, c1, a2, c2, M, asyn)
    ok1, ok2, oh, table = P.plan(a1, c1, a2, c2, M, asyn)
    assert h == pytest.approx(oh, rel=1e-12)
    assert P.parallel_dim_f(c1, k1, asyn) * k2 <= M
    assert table[(k1, k2)] == pytest.approx(oh, rel=1e-12)          # it is a maximiser
    ties = [kk for kk, v in table.items() if v >= oh * (1 - 1e-9)]
    assert (k1, k2) in ties
    # among maximisers: smallest k1, then smallest k2.  Checked whenever the oracle's maximisers are exactly equal
    # (async pairs beyond the depth limit are) or unique; two different pairs within 1e-9 of each other are left to
    # rounding
    if all(table[t] == oh for t in ties):
        assert (k1, k2) == min(ties) == (ok1, ok2)


def test_invalid_arguments():
    for a, c, k in ((0.0, 0.2, 3), (1.0, 0.2, 3), (0.5, 0.0, 3), (0.5, 1.0, 3), (0.5, 0.2, 0), (float("nan"), 0.2, 3)):
        for fn in (B.la_speedup_step_sync, B.la_speedup_step_async, B.la_speedup_token):
            with pytest.raises(B.LaError):
                fn(a, c, k)
    with pytest.raises(B.LaError):
        B.la_plan_budget(0.6, 0.2, 0.6, 0.1, 0, True)
    with pytest.raises(B.LaError):
        B.la_plan_budget(0.6, 1.2, 0.6, 0.1, 16, True)
