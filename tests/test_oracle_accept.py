"""Pins of the CPU oracle's token-level accept / resample (no GPU).

What fixes the expected values: the defining property of speculative sampling
(the emitted token is distributed as the target p, Section 2), the expected
number of emitted tokens (1-a^(K+1))/(1-a) (numerator of g, Section 2), the
acceptance probability sum(min(p,q)), and hand-computed small distributions.
"""
import math

import numpy as np
import pytest


def logits_of(p):
    p = np.asarray(p, dtype=np.float64)
    with np.errstate(divide="ignore"):
        return np.where(p > 0, np.log(np.maximum(p, 1e-300)), -1.0e4).astype(np.float32)


def run(oracle, t, d, tok, ua, us, **kw):
    return oracle.spec_accept(np.asarray(t, np.float32), np.asarray(d, np.float32), tok, ua, us, logits_dtype="f32",
                              **kw)


def chi2(counts, probs):
    n = counts.sum()
    keep = probs > 0
    assert counts[~keep].sum() == 0
    e = n * probs[keep]
    return float(((counts[keep] - e) ** 2 / e).sum())


def test_emitted_token_is_distributed_as_target(oracle):
    """V=8, K=1, 10^6 seeded trials with x ~ q: first emitted token ~ p_0, bonus ~ p_1, accept rate = sum min(p,q)."""
    rng = np.random.default_rng(2025)
    V, N = 8, 1_000_000
    t_row = rng.normal(0, 2, size=(2, V)).astype(np.float32)
    d_row = rng.normal(0, 2, size=(1, V)).astype(np.float32)
    p0 = np.exp(t_row[0].astype(np.float64)); p0 /= p0.sum()
    p1 = np.exp(t_row[1].astype(np.float64)); p1 /= p1.sum()
    q0 = np.exp(d_row[0].astype(np.float64)); q0 /= q0.sum()
    t = np.broadcast_to(t_row, (N, 2, V)).copy()
    d = np.broadcast_to(d_row, (N, 1, V)).copy()
    tok = rng.choice(V, size=(N, 1), p=q0).astype(np.int32)
    ua = rng.random((N, 1), dtype=np.float32)
    us = rng.random((N,), dtype=np.float32)
    r = run(oracle, t, d, tok, ua, us)
    n, nxt = r["accepted_len"], r["next_token"]
    assert set(np.unique(n)) <= {0, 1}
    first = np.where(n == 1, tok[:, 0], nxt)
    # chi-square, 7 degrees of freedom: P(chi2 > 29.9) ~ 1e-4
    assert chi2(np.bincount(first, minlength=V), p0) < 29.9
    assert chi2(np.bincount(nxt[n == 1], minlength=V), p1) < 29.9
    alpha = np.minimum(p0, q0).sum()
    assert abs((n == 1).mean() - alpha) < 4.5 * math.sqrt(alpha * (1 - alpha) / N)
    # a rejected draw never returns a token whose residual is zero
    resid = np.maximum(p0 - q0, 0)
    assert (resid[nxt[n == 0]] > 0).all()
    assert chi2(np.bincount(nxt[n == 0], minlength=V), resid / resid.sum()) < 29.9


def test_expected_emitted_length_follows_g_numerator(oracle):
    """K identical (p,q) positions, tokens iid from q => E[n+1] = (1-a^(K+1))/(1-a)."""
    rng = np.random.default_rng(7)
    V, K, N = 6, 4, 300_000
    p = np.array([0.35, 0.05, 0.2, 0.1, 0.25, 0.05])
    q = np.array([0.15, 0.25, 0.2, 0.2, 0.1, 0.1])
    t = np.broadcast_to(logits_of(p), (N, K + 1, V)).copy()
    d = np.broadcast_to(logits_of(q), (N, K, V)).copy()
    tok = rng.choice(V, size=(N, K), p=q).astype(np.int32)
    r = run(oracle, t, d, tok, rng.random((N, K), dtype=np.float32), rng.random((N,), dtype=np.float32))
    a = np.minimum(p, q).sum()
    expect = (1 - a ** (K + 1)) / (1 - a)
    emitted = r["accepted_len"].astype(np.float64) + 1
    assert abs(emitted.mean() - expect) < 4.5 * emitted.std() / math.sqrt(N)
    # geometric law of the accepted length
    for k in range(K):
        assert abs((r["accepted_len"] == k).mean() - a ** k * (1 - a)) < 5e-3
    assert abs((r["accepted_len"] == K).mean() - a ** K) < 5e-3


def test_hand_computed_residual_and_cdf(oracle):
    # p=[.6,.1,.3], q=[.2,.6,.2], x=1: ratio 1/6; residual [.4,0,.1] -> token 0 for u<.8 else 2
    p, q = [0.6, 0.1, 0.3], [0.2, 0.6, 0.2]
    us = np.array([0.0, 0.5, 0.79, 0.81, 0.999], dtype=np.float32)
    N = us.size
    t = np.broadcast_to(logits_of(p), (N, 2, 3)).copy()
    d = np.broadcast_to(logits_of(q), (N, 1, 3)).copy()
    tok = np.full((N, 1), 1, dtype=np.int32)
    r = run(oracle, t, d, tok, np.full((N, 1), 0.5, np.float32), us)
    np.testing.assert_array_equal(r["accepted_len"], 0)
    np.testing.assert_array_equal(r["next_token"], [0, 0, 0, 2, 2])
    np.testing.assert_allclose(r["ratio"][:, 0], 1 / 6, rtol=1e-6)
    np.testing.assert_allclose(r["margin"][:, 0], 0.5 - 1 / 6, rtol=1e-6)
    np.testing.assert_allclose(r["cdf_lo"], [0, 0, 0, 0.8, 0.8], atol=1e-6)
    np.testing.assert_allclose(r["cdf_hi"], [0.8, 0.8, 0.8, 1, 1], atol=1e-6)
    # same rows, u below the ratio: accepted, bonus token from the next target row p1=[.1,.2,.7]
    t[:, 1] = logits_of([0.1, 0.2, 0.7])
    r = run(oracle, t, d, tok, np.full((N, 1), 0.1, np.float32), np.array([0.05, 0.15, 0.29, 0.31, 0.9], np.float32))
    np.testing.assert_array_equal(r["accepted_len"], 1)
    np.testing.assert_array_equal(r["next_token"], [0, 1, 1, 2, 2])
    # x with p >= q is accepted for every u in [0,1)
    tok0 = np.zeros((N, 1), dtype=np.int32)
    r = run(oracle, t, d, tok0, np.full((N, 1), 0.999999, np.float32), us)
    np.testing.assert_array_equal(r["accepted_len"], 1)


def test_stops_at_first_rejection(oracle):
    # position 0 accept (p==q), position 1 reject (p(x)=0), position 2 would accept
    V, K = 4, 3
    same = logits_of([0.25, 0.25, 0.25, 0.25])
    t = np.stack([same, logits_of([0, 0.5, 0.5, 0]), same, same])[None]
    d = np.stack([same, logits_of([1.0, 0, 0, 0]), same])[None]
    tok = np.array([[2, 0, 1]], dtype=np.int32)
    r = run(oracle, t, d, tok, np.array([[0.9, 0.0, 0.0]], np.float32), np.array([0.6], np.float32))
    assert r["accepted_len"][0] == 1
    assert r["next_token"][0] == 2                       # residual = p_1 = [0,.5,.5,0], u=.6 -> token 2
    assert np.isnan(r["ratio"][0, 2]) and np.isinf(r["margin"][0, 2])   # position 2 never examined
    # u_sample = 0 must still return a token that has mass (token 0 has none here)
    r = run(oracle, t, d, tok, np.array([[0.9, 0.0, 0.0]], np.float32), np.array([0.0], np.float32))
    assert r["accepted_len"][0] == 1 and r["next_token"][0] == 1


def test_special_cases(oracle):
    rng = np.random.default_rng(3)
    V, K, N = 16, 5, 2000
    lg = rng.normal(0, 2, size=(N, K + 1, V)).astype(np.float32)
    tok = rng.integers(0, V, size=(N, K)).astype(np.int32)
    ua = rng.random((N, K), dtype=np.float32)
    us = rng.random((N,), dtype=np.float32)
    # p == q  => everything accepted
    r = run(oracle, lg, lg[:, :K].copy(), tok, ua, us)
    np.testing.assert_array_equal(r["accepted_len"], K)
    np.testing.assert_allclose(r["ratio"], 1.0, rtol=1e-12)
    # disjoint supports => nothing accepted, resample from p_0 itself
    t = lg.copy(); t[:, :, V // 2:] = -1.0e4
    d = lg[:, :K].copy(); d[:, :, :V // 2] = -1.0e4
    tok_hi = rng.integers(V // 2, V, size=(N, K)).astype(np.int32)
    r = run(oracle, t, d, tok_hi, ua, us)
    np.testing.assert_array_equal(r["accepted_len"], 0)
    assert (r["next_token"] < V // 2).all()
    p0 = np.exp(t[:, 0].astype(np.float64)); p0 /= p0.sum(-1, keepdims=True)
    cdf = np.cumsum(p0, axis=-1)
    expect = (cdf > us[:, None].astype(np.float64)).argmax(-1)
    assert (r["next_token"] == expect).mean() > 0.999    # summation order may flip a draw sitting on an edge
    # one-hot draft on x: accept probability p(x); on rejection x itself cannot come back
    d1 = np.full((N, K, V), -1.0e4, dtype=np.float32)
    np.put_along_axis(d1, tok[:, :, None].astype(np.int64), 0.0, axis=-1)
    r = run(oracle, lg, d1, tok, ua, us)
    p = np.exp(lg.astype(np.float64)); p /= p.sum(-1, keepdims=True)
    px0 = np.take_along_axis(p[:, 0], tok[:, :1].astype(np.int64), axis=-1)[:, 0]
    np.testing.assert_array_equal(r["accepted_len"] >= 1, ua[:, 0].astype(np.float64) < px0)
    rej = r["accepted_len"] < K
    rej_pos = r["accepted_len"][rej]
    assert (r["next_token"][rej] != tok[rej, rej_pos]).all()
    # u_accept == 0 accepts wherever p(x) > 0
    r = run(oracle, lg, lg[:, :K][:, ::-1].copy(), tok, np.zeros_like(ua), us)
    np.testing.assert_array_equal(r["accepted_len"], K)


def test_temperature_is_logit_scaling(oracle):
    rng = np.random.default_rng(4)
    V, K, N = 32, 3, 500
    t = rng.normal(0, 2, size=(N, K + 1, V)).astype(np.float32)
    d = (t[:, :K] + rng.normal(0, 1, size=(N, K, V))).astype(np.float32)
    tok = rng.integers(0, V, size=(N, K)).astype(np.int32)
    ua = rng.random((N, K), dtype=np.float32)
    us = rng.random((N,), dtype=np.float32)
    a = run(oracle, t, d, tok, ua, us, temperature=0.5)
    b = run(oracle, 2 * t, 2 * d, tok, ua, us, temperature=1.0)
    for k in ("accepted_len", "next_token", "ratio"):
        np.testing.assert_array_equal(a[k], b[k])
    c = run(oracle, t, d, tok, ua, us, temperature=1.0)
    assert not np.array_equal(a["ratio"], c["ratio"])


def test_bf16_storage_equals_widened_f32(oracle):
    from paper_2506_19830_amd import workloads as W
    case = W.AcceptCase("a", 6, 3, 300, "bf16", seed=5)
    inp = W.make_accept_inputs(case)
    a = oracle.spec_accept(**inp, logits_dtype="bf16")
    wide = dict(inp)
    wide["target_logits"] = oracle.widen(inp["target_logits"], "bf16").astype(np.float32)
    wide["draft_logits"] = oracle.widen(inp["draft_logits"], "bf16").astype(np.float32)
    b = oracle.spec_accept(**wide, logits_dtype="f32")
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])


def test_ratio_matches_independent_softmax(oracle):
    import torch
    from paper_2506_19830_amd import workloads as W
    case = W.AcceptCase("a", 5, 4, 1000, "f32", seed=6)
    inp = W.make_accept_inputs(case)
    r = oracle.spec_accept(**inp, logits_dtype="f32")
    lp = torch.log_softmax(torch.from_numpy(inp["target_logits"]).double(), -1)[:, :4]
    lq = torch.log_softmax(torch.from_numpy(inp["draft_logits"]).double(), -1)
    idx = torch.from_numpy(inp["draft_tokens"]).long()[..., None]
    ref = torch.exp(lp.gather(-1, idx) - lq.gather(-1, idx))[..., 0].numpy()
    seen = ~np.isnan(r["ratio"])
    assert seen[:, 0].all()
    np.testing.assert_allclose(r["ratio"][seen], ref[seen], rtol=1e-10)
    # accepted length is the first position whose uniform is not below min(1, ratio)
    ok = inp["u_accept"].astype(np.float64) < np.minimum(1.0, ref)
    expect = np.where(ok.all(1), 4, (~ok).argmax(1))
    np.testing.assert_array_equal(r["accepted_len"], expect)


def test_masked_logits_have_exactly_zero_mass(oracle):
    """-inf logits (a constrained vocabulary): the ratios equal an independent softmax over the unmasked entries, a
    drafted token the target masks is rejected, and over many draws no masked token is ever emitted while the
    emitted tokens follow the target restricted to its support."""
    import torch
    rng = np.random.default_rng(5)
    V, K, NB = 12, 1, 40000
    t1 = rng.normal(size=V).astype(np.float32)
    d1 = (t1 + rng.normal(scale=0.7, size=V)).astype(np.float32)
    t1[[2, 7]] = -np.inf                        # masked in the target: p = 0
    d1[[7, 9]] = -np.inf                        # masked in the draft: q = 0
    p = torch.softmax(torch.from_numpy(t1).double(), -1).numpy()
    q = torch.softmax(torch.from_numpy(d1).double(), -1).numpy()
    assert p[2] == 0 and p[7] == 0 and q[9] == 0
    tok = rng.choice(V, size=(NB, K), p=q).astype(np.int32)          # x ~ q: never 7 or 9
    t = np.tile(t1, (NB, K + 1, 1))
    d = np.tile(d1, (NB, K, 1))
    r = oracle.spec_accept(t, d, tok, rng.random((NB, K), dtype=np.float32), rng.random(NB, dtype=np.float32),
                           logits_dtype="f32")
    np.testing.assert_allclose(r["ratio"][:, 0], p[tok[:, 0]] / q[tok[:, 0]], rtol=1e-12)
    assert (r["accepted_len"][tok[:, 0] == 2] == 0).all()              # p(x) = 0: always rejected
    emitted = np.where(r["accepted_len"] >= 1, tok[:, 0], r["next_token"])
    counts = np.bincount(emitted, minlength=V)
    assert counts[2] == 0 and counts[7] == 0                           # no mass, never emitted
    keep = p > 0
    chi2 = (((counts[keep] - NB * p[keep]) ** 2) / (NB * p[keep])).sum()
    assert chi2 < 40.0                                                 # 9 degrees of freedom; P(chi2 > 40) < 1e-5


def test_rejects_bad_arguments(oracle):
    t = np.zeros((1, 2, 4), np.float32)
    d = np.zeros((1, 1, 4), np.float32)
    with pytest.raises(ValueError):
        run(oracle, t, d, np.array([[4]], np.int32), np.zeros((1, 1), np.float32), np.zeros((1,), np.float32))
    with pytest.raises(ValueError):
        run(oracle, t, d, np.array([[0]], np.int32), np.zeros((1, 1), np.float32), np.zeros((1,), np.float32),
            temperature=0.0)


# ------------------------------------------------------------------------------------------ point-mass draft
# Section 4 (Setup): the paper's token-level drafts come from prompt lookup (n-gram), which proposes tokens without a
# distribution: q_i is the point mass at x_i.  The rule of Section 2 then accepts with probability p_i(x_i) and
# resamples from p_n with x_n removed.

def run_onehot(oracle, t, tok, ua, us, **kw):
    return oracle.spec_accept(np.asarray(t, np.float32), None, tok, ua, us, logits_dtype="f32", **kw)


def test_point_mass_draft_emits_the_target_distribution(oracle):
    """V=8, K=1, a fixed drafted token: P(accept) = p(x); the emitted token is still distributed as p_0 (accepted
    x with probability p(x), otherwise y != x with probability (1-p(x)) * p(y)/(1-p(x)))."""
    rng = np.random.default_rng(77)
    V, N, x = 8, 600_000, 3
    t_row = rng.normal(0, 1.5, size=(2, V)).astype(np.float32)
    p0 = np.exp(t_row[0].astype(np.float64)); p0 /= p0.sum()
    p1 = np.exp(t_row[1].astype(np.float64)); p1 /= p1.sum()
    t = np.broadcast_to(t_row, (N, 2, V)).copy()
    tok = np.full((N, 1), x, dtype=np.int32)
    ua = rng.random((N, 1), dtype=np.float32)
    us = rng.random((N,), dtype=np.float32)
    r = run_onehot(oracle, t, tok, ua, us)
    n, nxt = r["accepted_len"], r["next_token"]
    assert abs((n == 1).mean() - p0[x]) < 4.5 * math.sqrt(p0[x] * (1 - p0[x]) / N)
    np.testing.assert_array_equal(n == 1, ua[:, 0].astype(np.float64) < p0[x])      # the test is u < p(x)
    assert (nxt[n == 0] != x).all()                                                  # x is removed from the residual
    first = np.where(n == 1, x, nxt)
    assert chi2(np.bincount(first, minlength=V), p0) < 29.9
    assert chi2(np.bincount(nxt[n == 1], minlength=V), p1) < 29.9
    rest = p0.copy(); rest[x] = 0
    assert chi2(np.bincount(nxt[n == 0], minlength=V), rest / rest.sum()) < 29.9
    np.testing.assert_allclose(r["ratio"][:, 0], p0[x], rtol=1e-12)


def test_point_mass_draft_equals_a_dense_draft_that_is_a_point_mass(oracle):
    """The same problem written with dense draft logits that put all mass on the drafted token (every other logit
    1e9 lower, so the fp64 softmax is exactly 0/1) must give identical results through the dense code path."""
    rng = np.random.default_rng(5)
    NB, K, V = 256, 5, 37
    t = rng.normal(0, 2.5, size=(NB, K + 1, V)).astype(np.float32)
    tok = rng.integers(0, V, size=(NB, K)).astype(np.int32)
    # make acceptance likely enough that all lengths 0..K occur
    for b in range(NB):
        for i in range(K):
            t[b, i, tok[b, i]] += 7.0
    ua = rng.random((NB, K), dtype=np.float32)
    us = rng.random((NB,), dtype=np.float32)
    d = np.full((NB, K, V), -1.0e9, dtype=np.float32)
    np.put_along_axis(d, tok[:, :, None], 0.0, axis=2)
    a = run_onehot(oracle, t, tok, ua, us)
    b_ = run(oracle, t, d, tok, ua, us)
    assert set(np.unique(a["accepted_len"])) == set(range(K + 1))
    for k in ("accepted_len", "next_token"):
        np.testing.assert_array_equal(a[k], b_[k])
    for k in ("ratio", "cdf_lo", "cdf_hi"):
        np.testing.assert_array_equal(np.nan_to_num(a[k], nan=-1.0), np.nan_to_num(b_[k], nan=-1.0))


def test_point_mass_draft_certain_token_is_always_accepted(oracle):
    V, K = 6, 3
    t = np.full((1, K + 1, V), -1.0e4, dtype=np.float32)
    tok = np.array([[2, 4, 1]], dtype=np.int32)
    for i in range(K):
        t[0, i, tok[0, i]] = 0.0
    t[0, K] = np.log(np.array([0.1, 0.2, 0.3, 0.15, 0.15, 0.1], dtype=np.float32))
    r = run_onehot(oracle, t, tok, np.array([[0.999, 0.5, 0.0]], np.float32), np.array([0.35], np.float32))
    assert r["accepted_len"][0] == K
    assert r["next_token"][0] == 2          # cumulative 0.1, 0.3, 0.6: first sum > 0.35 is token 2


# ------------------------------------------------------------------------------------------ top-k / top-p warping
# Section 4 (Setup): temperature 0.6, top_p 0.95 (and top_k 20 for one model family).  Order: temperature, top-k,
# top-p, renormalise.

def torch_warp(logits, temperature, top_k, top_p):
    """The same warp from library pieces (torch sort / topk / cumsum in fp64), written the way sampling code usually
    is: mask logits below the k-th largest, softmax, sort, drop a token when the mass in front of it reaches top_p."""
    import torch
    x = torch.as_tensor(np.asarray(logits, dtype=np.float64)) / temperature
    if 0 < top_k < x.numel():
        kth = torch.topk(x, top_k).values[-1]
        x = torch.where(x < kth, torch.full_like(x, -float("inf")), x)
    p = torch.softmax(x, dim=-1)
    if top_p < 1.0:
        sp, order = torch.sort(p, descending=True, stable=True)
        before = torch.cumsum(sp, dim=-1) - sp
        drop = before >= top_p
        p = p.clone()
        p[order[drop]] = 0.0
        p = p / p.sum()
    return p.numpy()


@pytest.mark.parametrize("top_k,top_p,temperature", [(20, 0.95, 0.6), (0, 0.95, 0.6), (20, 1.0, 1.0), (1, 1.0, 1.0),
                                                     (5, 0.5, 2.0), (0, 0.3, 1.0), (1000, 0.999, 0.6)])
def test_warp_matches_sort_based_reference(oracle, top_k, top_p, temperature):
    rng = np.random.default_rng(11)
    for V, std in ((1000, 3.0), (257, 1.0), (4096, 6.0)):
        logits = (rng.standard_normal(V) * std).astype(np.float32)     # continuous values: no ties
        got, margin = oracle.warp_probs(logits, logits_dtype="f32", temperature=temperature, top_k=top_k, top_p=top_p)
        ref = torch_warp(logits, temperature, top_k, top_p)
        np.testing.assert_array_equal(got > 0, ref > 0)
        np.testing.assert_allclose(got, ref, rtol=1e-12, atol=0)
        assert abs(got.sum() - 1.0) < 1e-12
        if top_p < 1.0:
            assert margin > 1e-9
        if 0 < top_k < V:
            assert (got > 0).sum() <= top_k


def test_warp_keeps_ties_together_and_special_cases(oracle):
    # values 5 > 3 = 3 = 3 > 1 > 0: top_k = 2 keeps the 5 and all three 3s
    logits = np.array([3.0, 5.0, 1.0, 3.0, 0.0, 3.0], dtype=np.float32)
    p, _ = oracle.warp_probs(logits, logits_dtype="f32", top_k=2)
    assert list(np.nonzero(p)[0]) == [0, 1, 3, 5]
    e = np.exp(logits.astype(np.float64) - 5.0)
    np.testing.assert_allclose(p[[0, 1, 3, 5]], e[[0, 1, 3, 5]] / e[[0, 1, 3, 5]].sum(), rtol=1e-14)
    # top_p: the 5 alone has mass 0.665 of the whole row: top_p = 0.6 keeps only it, 0.7 adds the tied group as a whole
    full = e / e.sum()
    assert 0.6 < full[1] < 0.7
    p6, _ = oracle.warp_probs(logits, logits_dtype="f32", top_p=0.6)
    assert list(np.nonzero(p6)[0]) == [1] and p6[1] == 1.0
    p7, _ = oracle.warp_probs(logits, logits_dtype="f32", top_p=0.7)
    assert list(np.nonzero(p7)[0]) == [0, 1, 3, 5]
    # off switches
    off, mg = oracle.warp_probs(logits, logits_dtype="f32", top_k=0, top_p=1.0)
    np.testing.assert_allclose(off, full, rtol=1e-14)
    assert mg == np.inf
    same, _ = oracle.warp_probs(logits, logits_dtype="f32", top_k=6, top_p=1.0)
    np.testing.assert_array_equal(same, off)
    # top-p is applied to what top-k kept: with k = 1 everything else is gone whatever top_p says
    g, _ = oracle.warp_probs(logits, logits_dtype="f32", top_k=1, top_p=0.01)
    assert list(np.nonzero(g)[0]) == [1]


def test_accept_with_warp_emits_the_warped_target(oracle):
    """V=12, K=1, dense draft, top_k=5, top_p=0.8, T=0.7: the emitted token follows the warped p_0 (speculative
    sampling is exact for whatever target distribution is plugged in), the bonus token the warped p_1."""
    rng = np.random.default_rng(99)
    V, N = 12, 600_000
    kw = dict(temperature=0.7, top_k=5, top_p=0.8)
    t_row = rng.normal(0, 1.5, size=(2, V)).astype(np.float32)
    d_row = rng.normal(0, 1.5, size=(1, V)).astype(np.float32)
    w0, _ = oracle.warp_probs(t_row[0], logits_dtype="f32", **kw)
    w1, _ = oracle.warp_probs(t_row[1], logits_dtype="f32", **kw)
    assert 1 < (w0 > 0).sum() < 5 and abs(w0.sum() - 1) < 1e-12      # both filters bite
    q0 = np.exp(d_row[0].astype(np.float64) / 0.7); q0 /= q0.sum()
    t = np.broadcast_to(t_row, (N, 2, V)).copy()
    d = np.broadcast_to(d_row, (N, 1, V)).copy()
    tok = rng.choice(V, size=(N, 1), p=q0).astype(np.int32)
    ua = rng.random((N, 1), dtype=np.float32)
    us = rng.random((N,), dtype=np.float32)
    r = run(oracle, t, d, tok, ua, us, **kw)
    n, nxt = r["accepted_len"], r["next_token"]
    first = np.where(n == 1, tok[:, 0], nxt)
    dof = int((w0 > 0).sum()) - 1
    assert chi2(np.bincount(first, minlength=V), w0) < 25.0 + 5 * dof      # generous 1e-4-level bound
    assert chi2(np.bincount(nxt[n == 1], minlength=V), w1) < 25.0 + 5 * int((w1 > 0).sum())
    alpha = np.minimum(w0, q0).sum()
    assert abs((n == 1).mean() - alpha) < 4.5 * math.sqrt(alpha * (1 - alpha) / N)
    assert (w0[first] > 0).all()                                            # nothing outside the kept set is emitted


def test_greedy_limit_with_point_mass_draft(oracle):
    """top_k = 1 makes the target a point mass at its argmax: a drafted token is accepted iff it is the argmax, and
    the extra token is the argmax of the row where the walk stopped."""
    rng = np.random.default_rng(4)
    NB, K, V = 300, 4, 50
    t = rng.normal(0, 2, size=(NB, K + 1, V)).astype(np.float32)
    am = t.argmax(-1)
    tok = np.where(rng.random((NB, K)) < 0.7, am[:, :K], rng.integers(0, V, size=(NB, K))).astype(np.int32)
    r = oracle.spec_accept(t, None, tok, rng.random((NB, K), dtype=np.float32), rng.random((NB,), dtype=np.float32),
                           logits_dtype="f32", top_k=1)
    match = tok == am[:, :K]
    n_ref = np.where(match.all(1), K, np.argmin(match, axis=1))
    np.testing.assert_array_equal(r["accepted_len"], n_ref)
    np.testing.assert_array_equal(r["next_token"], am[np.arange(NB), n_ref])
