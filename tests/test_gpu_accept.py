"""GPU parity of la_spec_accept against the CPU oracle, through the C ABI.

Bar: accepted lengths and token indices bit-exact for the fixed uniforms; branches whose decisive accept draw lies
within 1e-6 of the min(1, p/q) threshold (in the oracle's fp64) are counted and set aside, as the benchmark states.
"""
import numpy as np
import pytest

from paper_2506_19830_amd import workloads as W

pytestmark = pytest.mark.gpu


def check(oracle, case, max_near=None):
    from gpu_util import compare_accept, run_accept
    print(f"accept case {case.name} NB={case.NB} K={case.K} V={case.V} {case.logits_dtype} T={case.temperature}",
          flush=True)
    inp = W.make_accept_inputs(case)
    got = run_accept(case, inp)
    ref = oracle.spec_accept(**inp, logits_dtype=case.logits_dtype, temperature=case.temperature, top_k=case.top_k,
                             top_p=float(np.float32(case.top_p)))
    bad_n, bad_tok, near = compare_accept(got, ref)
    print(f"  near-threshold branches set aside: {near} of {case.NB}", flush=True)
    assert bad_n == 0, f"{bad_n} accepted lengths differ"
    assert bad_tok == 0, f"{bad_tok} tokens differ"
    if max_near is not None:
        assert near <= max_near
    examined = np.isfinite(ref["ratio"])
    np.testing.assert_allclose(got["ratio"][examined], ref["ratio"][examined], rtol=2e-4)
    assert (got["next_token"] >= 0).all() and (got["next_token"] < case.V).all()
    return got, ref


def test_config1_accept(oracle):
    _, case = W.config(1)
    check(oracle, case, max_near=0)


@pytest.mark.parametrize("case", [
    W.AcceptCase("many_small", 600, 4, 512, "f32", target_std=2.0, draft_noise_std=0.7, seed=1),
    W.AcceptCase("odd_vocab_f32", 64, 3, 1001, "f32", seed=2),          # rows not 16-byte aligned: scalar loads
    W.AcceptCase("odd_vocab_bf16", 64, 3, 8193, "bf16", seed=3),         # one full slice + 1 token
    W.AcceptCase("tiny_vocab", 200, 2, 3, "f32", target_std=1.0, draft_noise_std=0.5, seed=4),
    W.AcceptCase("two_slices_bf16", 50, 5, 16384, "bf16", seed=5),
    W.AcceptCase("temperature", 100, 4, 4096, "f32", temperature=0.6, seed=6),
    W.AcceptCase("k1", 128, 1, 2048, "bf16", seed=7),
    W.AcceptCase("long_draft", 3, 70, 700, "f32", target_std=1.0, draft_noise_std=0.05, seed=8),   # K > 64
], ids=lambda c: c.name)
def test_accept_edge_shapes(oracle, case):
    got, ref = check(oracle, case)
    if case.name == "many_small":
        # both outcomes are exercised
        assert (ref["accepted_len"] == case.K).any() and (ref["accepted_len"] == 0).any()


@pytest.mark.parametrize("n", [2, 3, 4, 5])
def test_accept_benchmark_configs(oracle, n):
    _, case = W.config(n)
    check(oracle, case)


def test_accept_is_deterministic():
    from gpu_util import run_accept
    case = W.AcceptCase("det", 16, 4, 50000, "bf16", seed=9)
    inp = W.make_accept_inputs(case)
    a, b = run_accept(case, inp), run_accept(case, inp)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])


def test_identical_models_accept_everything():
    from gpu_util import run_accept
    case = W.AcceptCase("same", 8, 6, 30000, "bf16", draft_noise_std=0.0, seed=10)
    inp = W.make_accept_inputs(case)
    got = run_accept(case, inp)
    np.testing.assert_array_equal(got["accepted_len"], case.K)
    np.testing.assert_allclose(got["ratio"], 1.0, rtol=1e-6)


def test_ratio_is_reported_at_every_position_also_behind_the_rejection(oracle):
    """accept_ratio holds p_i(x_i)/q_i(x_i) for every drafted position, not only the examined ones, also when the
    positions take several 64-position passes and the rejection lies in the first.  The oracle only evaluates what it
    examines, so its ratios come from a second run in which every draw accepts (u = 0); the ratio does not depend
    on the draw."""
    from gpu_util import run_accept
    for case in (W.AcceptCase("ratio_k70", 6, 70, 700, "f32", target_std=1.0, draft_noise_std=0.3, seed=41),
                 W.AcceptCase("ratio_k150", 4, 150, 3000, "bf16", target_std=2.0, draft_noise_std=0.5, seed=42),
                 W.AcceptCase("ratio_k9", 16, 9, 20000, "bf16", seed=43)):
        inp = W.make_accept_inputs(case)
        got = run_accept(case, inp)
        ref = oracle.spec_accept(**inp, logits_dtype=case.logits_dtype)
        every = dict(inp, u_accept=np.zeros_like(inp["u_accept"]))
        ref_all = oracle.spec_accept(**every, logits_dtype=case.logits_dtype)
        assert (ref_all["accepted_len"] == case.K).all()              # every position examined
        assert (ref["accepted_len"] < min(case.K, 64)).any()          # the real draws stop early somewhere
        np.testing.assert_array_equal(got["accepted_len"], ref["accepted_len"])
        np.testing.assert_array_equal(got["next_token"], ref["next_token"])
        assert np.isfinite(got["ratio"]).all()
        np.testing.assert_allclose(got["ratio"], ref_all["ratio"], rtol=2e-4)


def _mask_logits(case, inp, rng, frac, span, target_only_frac):
    """-inf logits: a constrained vocabulary (the same positions in the target and the draft rows: a random
    fraction plus one whole span), and some more positions in the target rows alone."""
    neg = {"f32": np.float32(-np.inf), "bf16": np.uint16(0xFF80)}[case.logits_dtype]
    both = rng.random(case.V) < frac
    both[span[0]:span[1]] = True
    both[rng.integers(0, case.V)] = False                        # never everything
    t, d = inp["target_logits"].copy(), None if inp["draft_logits"] is None else inp["draft_logits"].copy()
    t[:, :, both] = neg
    if d is not None:
        d[:, :, both] = neg
    only_t = (rng.random(t.shape) < target_only_frac) & ~both[None, None, :]
    t[only_t] = neg
    # every fourth branch: the target masks the first drafted token itself (p = 0 at a token the draft proposed)
    for nb in range(1, case.NB, 4):
        t[nb, 0, inp["draft_tokens"][nb, 0]] = neg
    return dict(inp, target_logits=t, draft_logits=d)


@pytest.mark.parametrize("case,span", [
    # a whole 16384-logit statistics slice of bf16 rows (and whole 2048-token slices of the fp64 path) masked
    (W.AcceptCase("masked_bf16", 24, 4, 40000, "bf16", seed=44), (16384, 32768)),
    # fp32: statistics slices hold 8192 logits
    (W.AcceptCase("masked_f32", 24, 3, 20000, "f32", seed=45), (8192, 16384)),
    (W.AcceptCase("masked_small", 64, 4, 700, "f32", target_std=1.5, seed=46), (100, 300)),
    (W.AcceptCase("masked_lookup_warped", 24, 4, 40000, "bf16", temperature=0.6, top_k=20, top_p=0.95,
                  point_mass=True, peak=9.0, seed=47), (16384, 32768)),
    (W.AcceptCase("masked_top_p", 12, 3, 40000, "bf16", temperature=0.8, top_p=0.9, seed=48), (16384, 32768)),
], ids=lambda x: getattr(x, "name", None))
def test_minus_infinity_logits(oracle, case, span):
    """Masked vocabulary entries (logit -inf) have probability exactly zero on both sides: they are never drawn, a
    drafted token the target masks is rejected (p = 0), one that both mask is rejected too (p = q = 0), whole
    statistics slices of -inf drop out of the row sums without a NaN."""
    from gpu_util import compare_accept, run_accept
    rng = np.random.default_rng(case.seed)
    inp = _mask_logits(case, W.make_accept_inputs(case), rng, 0.05, span, 0.02)
    got = run_accept(case, inp)
    ref = oracle.spec_accept(**inp, logits_dtype=case.logits_dtype, temperature=case.temperature, top_k=case.top_k,
                             top_p=float(np.float32(case.top_p)))
    bad_n, bad_tok, near = compare_accept(got, ref)
    assert bad_n == 0 and bad_tok == 0, f"{bad_n} lengths, {bad_tok} tokens differ ({near} set aside)"
    assert near <= 2
    examined = np.isfinite(ref["ratio"])
    np.testing.assert_allclose(got["ratio"][examined], ref["ratio"][examined], rtol=2e-4)
    # no returned token is a masked one
    t = inp["target_logits"]
    neg = t == ({"f32": np.float32(-np.inf), "bf16": np.uint16(0xFF80)}[case.logits_dtype])
    for nb in range(case.NB):
        assert not neg[nb, got["accepted_len"][nb], got["next_token"][nb]]
    # the walk met drafted tokens the target masks (p = 0: rejected on the spot) as well as ordinary ones
    assert (ref["accepted_len"][1::4] == 0).all()
    assert (ref["ratio"][examined] > 0).any()
    if not case.point_mass:
        assert (ref["accepted_len"] > 0).any()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_measure_zero_cases_of_the_accept_rule(oracle, dtype):
    """The cases the rule's wording leaves open, fixed by declaration and the same on both sides: q(x) = 0 < p(x)
    accepts whatever the draw; p(x) = q(x) = 0 rejects; a rejection after which the residual max(0, p - q) has no
    mass (p == q wherever either has mass) draws from p itself."""
    from gpu_util import run_accept
    V, K, NB = 8, 2, 4
    ninf = -np.inf
    base = np.array([0.5, -1.0, 2.0, 0.25, 1.5, -0.5, 0.0, 1.0], dtype=np.float32)
    t = np.tile(base, (NB, K + 1, 1))
    d = np.tile(base, (NB, K, 1))
    tok = np.zeros((NB, K), dtype=np.int32)
    # branch 0: token 3 has no draft mass, the target gives it some: accepted at any u; position 1 ordinary
    d[0, 0, 3] = ninf
    tok[0] = (3, 2)
    # branch 1: token 3 masked on both sides, the rows agree elsewhere: rejected, residual empty, drawn from p_0
    t[1, 0, 3] = ninf
    d[1, 0, 3] = ninf
    tok[1] = (3, 2)
    # branch 2: token 5 masked on both sides, rows differ: rejected, ordinary residual
    t[2, 0, 5] = ninf
    d[2, 0, 5] = ninf
    d[2, 0, :5] += np.float32(0.5)
    tok[2] = (5, 1)
    # branch 3: identical rows, nothing masked: everything accepted, bonus token from row K
    tok[3] = (2, 4)
    u_acc = np.array([[0.999, 0.1], [0.0, 0.5], [0.0, 0.5], [0.99, 0.99]], dtype=np.float32)
    u_smp = np.array([0.3, 0.77, 0.41, 0.05], dtype=np.float32)
    inp = {"target_logits": W.encode(t, dtype), "draft_logits": W.encode(d, dtype), "draft_tokens": tok,
           "u_accept": u_acc, "u_sample": u_smp}
    case = W.AcceptCase("measure_zero", NB, K, V, dtype)
    ref = oracle.spec_accept(**inp, logits_dtype=dtype)
    got = run_accept(case, inp)
    np.testing.assert_array_equal(ref["accepted_len"], [2, 0, 0, 2])
    np.testing.assert_array_equal(got["accepted_len"], ref["accepted_len"])
    np.testing.assert_array_equal(got["next_token"], ref["next_token"])
    assert got["next_token"][1] != 3 and got["next_token"][2] != 5      # a token without mass is never drawn
    assert np.isinf(got["ratio"][0, 0]) and np.isnan(got["ratio"][1, 0])  # p/q as computed: x/0 and 0/0


# ------------------------------------------------------------------------------------------ point-mass draft
POINT_MASS_CASES = [
    W.AcceptCase("pm_small", 400, 4, 512, "f32", target_std=2.0, point_mass=True, peak=7.0, seed=11),
    W.AcceptCase("pm_odd_vocab", 64, 3, 8193, "bf16", point_mass=True, peak=12.0, seed=12),
    W.AcceptCase("pm_k1_tiny", 200, 1, 3, "f32", target_std=1.0, point_mass=True, peak=1.0, seed=13),
    W.AcceptCase("pm_temperature", 100, 4, 4096, "f32", temperature=0.6, point_mass=True, peak=6.0, seed=14),
    W.AcceptCase("pm_long_draft", 3, 70, 700, "f32", target_std=1.0, point_mass=True, peak=12.0, seed=15),
    # the paper's setting at full vocabulary: 8 drafted tokens, temperature 0.6
    W.AcceptCase("pm_vocab152k_k8", 8, 8, 152064, "bf16", temperature=0.6, point_mass=True, peak=11.0, seed=16),
    W.AcceptCase("pm_vocab152k_k8_nb32", 32, 8, 152064, "bf16", point_mass=True, seed=17),
]


@pytest.mark.parametrize("case", POINT_MASS_CASES, ids=lambda c: c.name)
def test_point_mass_draft(oracle, case):
    """draft_logits = NULL: q is the point mass at the drafted token (prompt-lookup drafts).  Accept iff u < p(x);
    after a rejection the token comes from p with x removed, so it can never be x."""
    got, ref = check(oracle, case)
    inp = W.make_accept_inputs(case)
    rejected = got["accepted_len"] < case.K
    x_n = inp["draft_tokens"][np.arange(case.NB)[rejected], got["accepted_len"][rejected]]
    assert (got["next_token"][rejected] != x_n).all()
    if case.name in ("pm_small", "pm_vocab152k_k8_nb32"):
        assert (ref["accepted_len"] > 0).any() and (ref["accepted_len"] < case.K).any()


# ------------------------------------------------------------------------------------------ top-k / top-p warping
WARP_CASES = [
    W.AcceptCase("warp_small_dense", 300, 4, 512, "f32", target_std=2.0, draft_noise_std=0.7, temperature=0.6, top_k=20,
                 top_p=0.95, seed=21),
    W.AcceptCase("warp_topp_only", 100, 3, 4096, "f32", temperature=0.6, top_p=0.95, seed=22),
    W.AcceptCase("warp_topk_only_bf16", 64, 3, 8193, "bf16", top_k=20, seed=23),          # bf16: many tied logits
    W.AcceptCase("warp_greedy", 200, 4, 1000, "f32", top_k=1, point_mass=True, peak=3.0, seed=24),
    W.AcceptCase("warp_tiny_vocab", 200, 2, 3, "f32", target_std=1.0, draft_noise_std=0.5, top_k=2, top_p=0.7, seed=25),
    W.AcceptCase("warp_k_above_vocab", 50, 2, 100, "f32", top_k=500, top_p=0.9, seed=26),
    # the two settings of the paper's runs at full vocabulary, prompt-lookup drafts: (T 0.6, top_p 0.95, top_k 20)
    # and (T 0.6, top_p 0.95)
    W.AcceptCase("warp_qwen3_setting", 8, 8, 152064, "bf16", temperature=0.6, top_k=20, top_p=0.95, point_mass=True,
                 peak=11.0, seed=27),
    W.AcceptCase("warp_r1_setting", 8, 8, 152064, "bf16", temperature=0.6, top_p=0.95, point_mass=True, peak=11.0,
                 seed=28),
    W.AcceptCase("warp_dense_152k_f32", 4, 4, 152064, "f32", temperature=0.6, top_k=20, top_p=0.95, seed=29),
    # top-p alone on fp32 logits and dense drafts at full vocabulary (the slice-sum kernel and the 32-bit key search)
    W.AcceptCase("warp_topp_152k_f32", 4, 4, 152064, "f32", temperature=0.6, top_p=0.95, seed=30),
    W.AcceptCase("warp_topp_flat_152k_bf16", 4, 3, 152064, "bf16", target_std=1.0, temperature=1.0, top_p=0.9, seed=34),
]


@pytest.mark.parametrize("case", WARP_CASES, ids=lambda c: c.name)
def test_warped_target(oracle, case):
    """Temperature, top-k and top-p applied to the target rows before the accept rule (Section 4, Setup)."""
    got, ref = check(oracle, case)
    inp = W.make_accept_inputs(case)
    # the extra token always lies in the kept set of the row it was drawn from
    for nb in range(min(case.NB, 16)):
        n = int(ref["accepted_len"][nb])
        row = inp["target_logits"][nb, n]
        p, _ = oracle.warp_probs(row, logits_dtype=case.logits_dtype, temperature=case.temperature, top_k=case.top_k,
                                 top_p=float(np.float32(case.top_p)))
        assert p[got["next_token"][nb]] > 0


def check_inputs(oracle, case, inp):
    from gpu_util import compare_accept, run_accept
    got = run_accept(case, inp)
    ref = oracle.spec_accept(**inp, logits_dtype=case.logits_dtype, temperature=case.temperature, top_k=case.top_k,
                             top_p=float(np.float32(case.top_p)))
    bad_n, bad_tok, near = compare_accept(got, ref)
    print(f"  {case.name}: near-threshold branches set aside: {near} of {case.NB}", flush=True)
    assert bad_n == 0 and bad_tok == 0, f"{bad_n} accepted lengths, {bad_tok} tokens differ"
    assert near <= 2 + case.NB // 50      # a draw within 1e-6 of its threshold is a one-in-a-million event per position
    return got, ref


def test_warp_large_top_k(oracle):
    """A top_k above what the candidate-list path of the warp kernel takes: the histogram selection runs."""
    check(oracle, W.AcceptCase("warp_topk_200", 40, 3, 4096, "f32", temperature=0.8, top_k=200, top_p=0.9, seed=31))
    check(oracle, W.AcceptCase("warp_topk_129_bf16", 24, 2, 20000, "bf16", top_k=129, top_p=0.97, seed=32))
    check(oracle, W.AcceptCase("warp_topk_128_bf16", 24, 2, 20000, "bf16", top_k=128, top_p=0.97, seed=33))


@pytest.mark.parametrize("std,top_k,dtype", [(3.0, 20, "bf16"), (3.0, 20, "f32"), (0.5, 50, "bf16"), (0.5, 50, "f32"),
                                             (0.0, 5, "f32"), (3.0, 0, "bf16"), (3.0, 0, "f32"), (0.5, 0, "f32"),
                                             (0.0, 0, "bf16")])
def test_warp_tied_logits(oracle, std, top_k, dtype):
    """Target logits rounded to whole numbers, so that many tokens tie at every value: ties with the k-th largest
    value all stay, and a value group stays or goes as one under top-p.  With std 3 the candidate list of the warp
    kernel holds a few hundred tied keys; with std 0.5 the k-th value is shared by thousands of tokens, more than the
    list takes, and with std 0 by the whole row: the histogram path takes over.  top_k 0: top-p alone, whose
    candidate list is proposed by an fp32 histogram and checked exactly."""
    case = W.AcceptCase(f"warp_ties_{std}_{top_k}_{dtype}", 12, 3, 20000, dtype, target_std=max(std, 1.0),
                        temperature=0.7, top_k=top_k, top_p=0.9, point_mass=True, peak=0.0, seed=int(40 + std * 10))
    inp = W.make_accept_inputs(case)
    x = W._decode_for_sampling(inp["target_logits"], dtype)
    x = np.rint(x * (std / max(std, 1.0)))
    x[:, :, ::2] += 0.0          # every other zero a negative zero: the same value as +0 for both filters
    inp["target_logits"] = W.encode(x.astype(np.float32), dtype)
    got, ref = check_inputs(oracle, case, inp)
    # what was drawn has mass under the warped row
    for nb in range(case.NB):
        n = int(ref["accepted_len"][nb])
        p, _ = oracle.warp_probs(inp["target_logits"][nb, n], logits_dtype=dtype, temperature=case.temperature,
                                 top_k=case.top_k, top_p=float(np.float32(case.top_p)))
        assert p[got["next_token"][nb]] > 0


def random_warp_case(idx):
    rng = np.random.default_rng(7000 + idx)
    V = int(rng.choice([1000, 6000, 8192, 20000, 50257, 152064]))
    K = int(rng.choice([1, 2, 4]))
    NB = int(rng.choice([2, 5, 12])) if V <= 20000 else int(rng.choice([1, 3]))
    top_k = int(rng.choice([0, 0, 3, 64, 128, 129, 1000]))
    top_p = float(rng.choice([1.0, 0.999, 0.95, 0.7, 0.3, 0.05]))
    if top_k == 0 and top_p == 1.0:
        top_p = 0.9
    return W.AcceptCase(f"rand_warp{idx}", NB, K, V, str(rng.choice(["f32", "bf16"])),
                        target_std=float(rng.choice([0.5, 1.0, 3.0, 6.0])),
                        draft_noise_std=float(rng.choice([0.3, 1.0])),
                        temperature=float(rng.choice([1.0, 0.6, 1.5, 0.3])), seed=7000 + idx, top_k=top_k, top_p=top_p,
                        point_mass=bool(rng.integers(0, 2)), peak=float(rng.choice([0.0, 4.0, 9.0])))


@pytest.mark.parametrize("idx", range(28))
def test_warp_random_settings(oracle, idx):
    """Vocabulary, dtype, spread of the logits (a flat row keeps thousands of tokens under top-p, a peaked one a
    handful), temperature, top_k on both sides of the candidate-list limit and top_p from nearly nothing to nearly
    everything, drawn at random: whichever form of the warp kernel a row takes, the result is the oracle's."""
    case = random_warp_case(idx)
    print(f"  top_k={case.top_k} top_p={case.top_p} std={case.target_std} T={case.temperature} "
          f"point_mass={case.point_mass}", flush=True)
    check(oracle, case)


@pytest.mark.parametrize("case", [
    W.AcceptCase("huge_vocab_dense", 2, 2, 600_000, "bf16", seed=51),                       # 293 fine slices
    W.AcceptCase("max_vocab_dense", 1, 1, 1 << 21, "f32", seed=52),                         # 1024 fine slices: the limit
    # nine rows of 256 statistics slices: more than a workgroup of the decide kernel stages in LDS at once
    W.AcceptCase("max_vocab_dense_k4", 1, 4, 1 << 21, "f32", draft_noise_std=0.3, seed=55),
    W.AcceptCase("max_vocab_lookup_topk", 1, 2, 1 << 21, "bf16", temperature=0.6, top_k=20, top_p=0.95,
                 point_mass=True, peak=9.0, seed=53),
    W.AcceptCase("huge_vocab_lookup_topp", 2, 1, 600_000, "f32", temperature=0.6, top_p=0.9, point_mass=True,
                 peak=9.0, seed=54),
], ids=lambda c: c.name)
def test_accept_largest_vocabularies(oracle, case):
    """Vocabularies with more fine slices than a workgroup has lanes, up to the largest one the library takes: the
    folds and scans over the slice sums then run several terms per lane."""
    check(oracle, case)


def test_vocabulary_above_the_limit_is_refused():
    from paper_2506_19830_amd import binding as B
    desc = B.make_accept_desc(num_branches=1, num_draft=1, vocab=(1 << 21) + 1, logits_dtype="bf16")
    with pytest.raises(B.LaError):
        B.la_spec_accept_workspace(desc)


# ------------------------------------------------------------------------------------------ random shapes

def random_accept_case(idx):
    rng = np.random.default_rng(3000 + idx)
    V = int(rng.choice([2, 7, 64, 511, 1000, 4097, 8191, 8192, 8200, 16385, 32000, 50257, 100003, 151936, 152064]))
    K = int(rng.choice([1, 2, 3, 5, 8, 13]))
    NB = int(rng.choice([1, 2, 5, 16, 33, 100]))
    while NB * (2 * K + 1) * V > 12_000_000 and NB > 1:             # keeps the oracle quick
        NB = max(1, NB // 2)
    while (2 * K + 1) * V > 12_000_000:
        K = max(1, K // 2)
    point_mass = bool(rng.integers(0, 3) == 0)
    top_k = int(rng.choice([0, 0, 1, 5, 20, 50]))
    top_p = float(rng.choice([1.0, 1.0, 0.95, 0.8, 0.5]))
    return W.AcceptCase(f"rand_accept{idx}", NB, K, V, str(rng.choice(["f32", "bf16"])),
                        target_std=float(rng.choice([1.0, 2.0, 3.0])),
                        draft_noise_std=float(rng.choice([0.1, 0.5, 1.0])),
                        temperature=float(rng.choice([1.0, 0.6, 1.5])), seed=3000 + idx, top_k=top_k, top_p=top_p,
                        point_mass=point_mass, peak=float(rng.choice([2.0, 6.0, 11.0])))


@pytest.mark.parametrize("idx", range(24))
def test_accept_random_shapes(oracle, idx):
    """Branch count, draft length, vocabulary (around the slice and vector sizes and the real ones), dtype,
    temperature, top-k / top-p and dense or point-mass drafts drawn at random, each against the oracle."""
    case = random_accept_case(idx)
    print(f"  top_k={case.top_k} top_p={case.top_p} point_mass={case.point_mass}", flush=True)
    check(oracle, case)
