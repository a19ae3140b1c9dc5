"""GPU parity of la_verify_attention against the CPU oracle, through the C ABI.

Bar: max over output rows of  max|o - o*| / max|o*|  <= 1e-5 for fp32 tensors and <= 2e-2 for bf16 / fp8-KV
tensors (the benchmark's stated tolerance), on the same seeded inputs.
"""
from dataclasses import replace

import numpy as np
import pytest

from paper_2506_19830_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-5
TOL_LOWP = 2e-2


def oracle_attention(oracle, case, inp, row_ids=None, scale=None):
    return oracle.verify_attention(**inp, q_dtype=case.q_dtype, kv_dtype=case.kv_dtype,
                                   branch_kv_dtype=case.branch_kv_dtype, block_size=case.block_size,
                                   scale=case.scale if scale is None else scale, row_ids=row_ids)


def check_full(oracle, case, tol, kv_split_tokens=0, lse_tol=None):
    from gpu_util import error_report, row_errors, run_attention
    print(f"case {case.name} prefix={case.prefix_lens} gamma={case.gamma} L={case.L} Hq={case.Hq} Hkv={case.Hkv} "
          f"D={case.D} kv={case.kv_dtype} br={case.branch_kv_dtype} paged={case.paged} split={kv_split_tokens}",
          flush=True)
    inp = W.make_attention_inputs(case)
    got, lse = run_attention(case, inp, kv_split_tokens)
    ref, ref_lse = oracle_attention(oracle, case, inp)
    assert np.isfinite(got).all()
    err = row_errors(got, ref)
    print(f"  errors: {error_report(got, ref)}", flush=True)
    assert err.max() <= tol, f"max row error {err.max():.3e} at row {err.argmax()}"
    # bf16 path: Q is rounded to bf16 once more after the score scale is folded into it, which moves every score by
    # up to 2^-9 of sum|q_d k_d|*scale (about 1e-3 rms, a few 1e-3 at worst for these inputs); LSE inherits that
    lse_tol = lse_tol if lse_tol is not None else (1e-5 if tol == TOL_F32 else 1e-2)
    assert np.abs(lse - ref_lse).max() <= lse_tol
    return got, ref


# ----------------------------------------------------------------------------------------- fp32 path

def test_config1_fp32(oracle):
    case, _ = W.config(1)
    check_full(oracle, case, TOL_F32)


@pytest.mark.parametrize("case", [
    W.AttnCase("f32_d128_ragged", (77, 0, 130), 3, 5, 6, 2, 128, "f32", "f32", "f32", "f32"),
    W.AttnCase("f32_paged", (300, 45), 2, 9, 8, 2, 64, "f32", "f32", "f32", "f32", paged=True, seed=2),
    W.AttnCase("f32_d256_block32", (100,), 2, 3, 2, 1, 256, "f32", "f32", "f32", "f32", block_size=32, seed=3),
    W.AttnCase("f32_no_prefix", (0,), 2, 70, 2, 2, 64, "f32", "f32", "f32", "f32", seed=4),
], ids=lambda c: c.name)
def test_fp32_edge_shapes(oracle, case):
    check_full(oracle, case, TOL_F32)


# ----------------------------------------------------------------------------------------- MFMA path

MFMA_CASES = [
    # several row tiles with a ragged last one (R = 3*20*8 = 480), prefix not a multiple of the 64-key tile
    W.AttnCase("bf16_ragged", (1000,), 3, 20, 16, 2, 128, seed=1),
    # branches longer than one key tile, row tiles straddling branches (L*G = 70*3 = 210)
    W.AttnCase("bf16_long_branch", (130,), 4, 70, 6, 2, 128, seed=2),
    # paged, several requests, empty and tiny prefixes, partly filled last block
    W.AttnCase("bf16_paged_multi", (777, 0, 5, 2049), 2, 17, 8, 2, 128, paged=True, seed=3),
    W.AttnCase("fp8_kv", (900,), 3, 33, 10, 2, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16", seed=4),
    W.AttnCase("fp8_kv_bf16_branch", (515, 64), 2, 40, 8, 1, 128, "bf16", "fp8_e4m3", "bf16", "f32", paged=True,
               seed=5),
    W.AttnCase("bf16_single_token_branches", (321,), 8, 1, 40, 8, 128, seed=6),
    W.AttnCase("bf16_block64", (700,), 2, 8, 4, 4, 128, block_size=64, paged=True, seed=7),
]


@pytest.mark.parametrize("case", MFMA_CASES, ids=lambda c: c.name)
@pytest.mark.parametrize("split", [0, 64, 256])
def test_mfma_small_cases(oracle, case, split):
    check_full(oracle, case, TOL_LOWP, kv_split_tokens=split)


@pytest.mark.parametrize("shape", [0, 1])
@pytest.mark.parametrize("case", [MFMA_CASES[0], MFMA_CASES[2], MFMA_CASES[3], MFMA_CASES[5]], ids=lambda c: c.name)
def test_every_kernel_shape(oracle, case, shape, monkeypatch):
    """The planner picks one of the kernel's (wavefronts, row blocks, LDS stages) shapes by a cost model; here
    each is forced in turn (the descriptor's kernel_shape field), with long and short chunks
    (odd and even tile counts per chunk, chunks shorter than the prefetch distance)."""
    monkeypatch.setattr("gpu_util.KERNEL_SHAPE", shape + 1)
    for split in (0, 64, 192, 320):
        check_full(oracle, case, TOL_LOWP, kv_split_tokens=split)


STREAM_CASES = [
    # few rows per KV head (the regime the streaming shapes are for): R = 8*1*5 = 40, 6*9*5 = 270, ragged prefixes
    W.AttnCase("fp8_stream_l1", (1000,), 8, 1, 40, 8, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16", seed=71),
    W.AttnCase("fp8_stream_paper_step", (2077,), 6, 9, 40, 8, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16", seed=72),
    # paged, several requests with empty / tiny / ragged prefixes, fp32 out, branches longer than a key tile
    W.AttnCase("fp8_stream_paged_multi", (777, 0, 5, 2049), 2, 17, 8, 2, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "f32",
               paged=True, seed=73),
    W.AttnCase("fp8_stream_long_branch", (130,), 2, 150, 4, 2, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16", seed=74),
    W.AttnCase("fp8_stream_block64", (700,), 2, 8, 4, 4, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16", block_size=64,
               paged=True, seed=75),
    W.AttnCase("fp8_stream_no_prefix", (0,), 3, 70, 2, 2, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16", seed=76),
]


@pytest.mark.parametrize("shape", [2, 3, 4])
@pytest.mark.parametrize("case", STREAM_CASES, ids=lambda c: c.name)
def test_every_streaming_shape(oracle, case, shape, monkeypatch):
    """The streaming shapes (direct global -> LDS loads, transposing LDS reads, row blocks x key slices) forced in
    turn: automatic chunking, one tile per chunk, chunks whose tile count is odd / not a multiple of the key
    slices / shorter than the prefetch depth."""
    monkeypatch.setattr("gpu_util.KERNEL_SHAPE", shape + 1)
    for split in (0, 64, 192, 320, 1024):
        check_full(oracle, case, TOL_LOWP, kv_split_tokens=split)


@pytest.mark.parametrize("shape", [0, 1])
@pytest.mark.parametrize("case", STREAM_CASES[:2], ids=lambda c: c.name)
def test_row_tile_shapes_with_idle_wavefronts(oracle, case, shape, monkeypatch):
    """Few rows on the row-tile shapes: wavefronts whose rows lie past R only stage tiles, in loops of their own
    (R = 40: one computing wavefront; R = 270: a last row tile with 14 rows).  Chunks of one to seven full tiles
    and the whole prefix, so that the steady-state loops and their tails run with every remainder."""
    monkeypatch.setattr("gpu_util.KERNEL_SHAPE", shape + 1)
    for split in (0, 64, 128, 192, 256, 320, 384, 448):
        check_full(oracle, case, TOL_LOWP, kv_split_tokens=split)


def _as_bf16(case, name):
    import dataclasses
    return dataclasses.replace(case, name=name, kv_dtype="bf16", branch_kv_dtype="bf16")


STREAM16_CASES = [_as_bf16(c, c.name.replace("fp8_", "bf16_")) for c in STREAM_CASES] + [
    # many rows per KV head (what these shapes are for): R = 8*16*4 = 512 spans two 256-row workgroups, ragged
    W.AttnCase("bf16_stream_rows512", (1500, 300), 8, 16, 8, 2, 128, "bf16", "bf16", "bf16", "bf16", paged=True,
               seed=77),
]


@pytest.mark.parametrize("shape", [5, 6])
@pytest.mark.parametrize("case", STREAM16_CASES, ids=lambda c: c.name)
def test_every_bf16_streaming_shape(oracle, case, shape, monkeypatch):
    """The streaming shapes for a bf16 cache (no conversion anywhere; transposing 16-bit LDS reads), forced."""
    monkeypatch.setattr("gpu_util.KERNEL_SHAPE", shape + 1)
    for split in (0, 64, 192, 320, 1024):
        check_full(oracle, case, TOL_LOWP, kv_split_tokens=split)


@pytest.mark.parametrize("shape,kv", [(0, "fp8_e4m3"), (1, "fp8_e4m3"), (2, "fp8_e4m3"), (3, "fp8_e4m3"), (4, "fp8_e4m3"),
                                      (0, "bf16"), (1, "bf16"), (5, "bf16"), (6, "bf16")])
@pytest.mark.parametrize("shift", [9.0, 45.0])
def test_running_maximum_that_jumps_late(oracle, shape, kv, shift, monkeypatch):
    """Scores that jump by `shift` nats (13 and 65 log2 units) somewhere behind the first key tile: inside the first
    tile's second key block, on a tile boundary, inside a later tile, and in the branch keys only.  The unmasked tiles
    of every kernel shape form their probabilities against a base that is only moved on a rare path (a row sum above a
    trigger: the block is redone, the maximum raised, the accumulators rescaled); N(0,1) scores never take that path
    after the first tile, these do -- once by a little (probabilities up to 2^13 before the trigger's threshold is
    met in the next block) and once by more than an fp32 exponential would survive without it.  The shift is common
    to all late keys, so its own rounding error (2^-9 of 45 nats) cancels in the output; the log-sum-exp carries it."""
    monkeypatch.setattr("gpu_util.KERNEL_SHAPE", shape + 1)
    for i, (prefix, late_from) in enumerate((((1000,), 40), ((1000,), 64), ((2077, 333), 300), ((130,), 10 ** 6))):
        case = W.AttnCase(f"late_jump_{late_from}", prefix, 6, 9, 40, 8, 128, "bf16", kv, kv, "bf16", paged=(i == 2),
                          seed=90 + i, late_key_shift=shift, late_from=late_from)
        for split in (0, 192):
            check_full(oracle, case, TOL_LOWP, kv_split_tokens=split, lse_tol=0.1)


@pytest.mark.parametrize("shape,case", [(s, c) for s in (2, 3, 4) for c in STREAM_CASES] +
                         [(s, c) for s in (5, 6) for c in STREAM16_CASES], ids=lambda v: getattr(v, "name", str(v)))
def test_second_attempt_of_the_streaming_shapes(oracle, case, shape, monkeypatch):
    """The streaming shapes reduce a chunk a second time, in a general form, when a score lies far above the base
    its unmasked tiles started from.  The benchmark library can make every workgroup do so: same bar against the
    oracle, and within rounding of what the first attempt gives on the same inputs."""
    from gpu_util import row_errors, run_attention
    from paper_2506_19830_amd import binding as B
    monkeypatch.setattr("gpu_util.KERNEL_SHAPE", shape + 1)
    inp = W.make_attention_inputs(case)
    ref, ref_lse = oracle_attention(oracle, case, inp)
    B.select_library("bench")
    try:
        for split in (0, 192):
            first, lse1 = run_attention(case, inp, split)
            B.la_selftest_second_attempt(True)
            try:
                second, lse2 = run_attention(case, inp, split)
            finally:
                B.la_selftest_second_attempt(False)
            assert np.isfinite(second).all()
            assert row_errors(second, ref).max() <= TOL_LOWP and np.abs(lse2 - ref_lse).max() <= 1e-2
            assert row_errors(second, first).max() <= TOL_LOWP
            assert not np.array_equal(second, first) or case.prefix_lens == (0,)   # (another summation order: the hook is live)
    finally:
        B.select_library("product")


def test_streaming_shape_is_refused_where_it_cannot_run(monkeypatch):
    from gpu_util import run_attention
    from paper_2506_19830_amd import binding as B
    monkeypatch.setattr("gpu_util.KERNEL_SHAPE", 3)
    case = MFMA_CASES[0]                                    # bf16 cache: no fp8 streaming shape
    with pytest.raises(B.LaError) as e:
        run_attention(case, W.make_attention_inputs(case))
    assert e.value.status == 2
    monkeypatch.setattr("gpu_util.KERNEL_SHAPE", 6)
    case = STREAM_CASES[0]                                  # fp8 cache: no bf16 streaming shape
    with pytest.raises(B.LaError) as e:
        run_attention(case, W.make_attention_inputs(case))
    assert e.value.status == 2


# ----------------------------------------------------------------------------------------- other head dimensions

GENERAL_CASES = [
    # bf16 / fp8 storage at head dimensions 64 and 256: the general kernel (fp32 arithmetic on exactly widened inputs)
    W.AttnCase("bf16_d64_paged", (300, 17), 3, 5, 8, 2, 64, "bf16", "bf16", "bf16", "bf16", paged=True, seed=81),
    W.AttnCase("fp8_d64", (515,), 2, 9, 6, 2, 64, "bf16", "fp8_e4m3", "fp8_e4m3", "f32", seed=82),
    W.AttnCase("fp8_bf16_branch_d256", (130,), 2, 4, 4, 1, 256, "bf16", "fp8_e4m3", "bf16", "bf16", seed=83),
    W.AttnCase("bf16_d256_no_prefix", (0,), 2, 70, 2, 2, 256, "bf16", "bf16", "bf16", "f32", seed=84),
]


@pytest.mark.parametrize("case", GENERAL_CASES, ids=lambda c: c.name)
def test_other_head_dimensions(oracle, case):
    """Inputs are widened exactly and everything is fp32, so with fp32 output the result is fp32-accurate; with bf16
    output the only rounding is the output's own."""
    from paper_2506_19830_amd import binding as B
    desc_plan = B.la_verify_attention_plan(
        B.make_attn_desc(num_requests=case.B, num_q_heads=case.Hq, num_kv_heads=case.Hkv, head_dim=case.D,
                         gamma=case.gamma, branch_len=case.L, block_size=case.block_size,
                         max_blocks_per_request=case.max_blocks, q_dtype=case.q_dtype, kv_dtype=case.kv_dtype,
                         branch_kv_dtype=case.branch_kv_dtype, out_dtype=case.out_dtype, softmax_scale=case.scale),
        [int(x) for x in case.prefix_lens])
    assert desc_plan["path"] == 1
    tol = 1e-5 if case.out_dtype == "f32" else 5e-3
    check_full(oracle, case, tol, lse_tol=1e-5)


def test_other_head_dimensions_nested_and_tree(oracle):
    check_nested(oracle, GENERAL_CASES[1], 40, 1e-5)
    check_tree(oracle, GENERAL_CASES[0], 2, 3, 6, 5e-3)


# ----------------------------------------------------------------------------------------- nested branches

def check_nested(oracle, case, chain_len, tol, chain_vis=None, kv_split_tokens=0):
    from gpu_util import row_errors, run_attention_nested
    inp = W.make_attention_inputs(case)
    chain = W.make_chain_inputs(case, chain_len, inp, chain_vis)
    print(f"nested case {case.name} prefix={case.prefix_lens} gamma={case.gamma} L={case.L} C={chain_len} "
          f"vis={chain['chain_vis'].tolist()} kv={case.kv_dtype} br={case.branch_kv_dtype} split={kv_split_tokens}",
          flush=True)
    got, lse = run_attention_nested(case, inp, chain, kv_split_tokens)
    ref, ref_lse = oracle.verify_attention(**inp, **chain, q_dtype=case.q_dtype, kv_dtype=case.kv_dtype,
                                           branch_kv_dtype=case.branch_kv_dtype, block_size=case.block_size,
                                           scale=case.scale)
    assert np.isfinite(got).all()
    err = row_errors(got, ref)
    assert err.max() <= tol, f"max row error {err.max():.3e} at row {err.argmax()}"
    assert np.abs(lse - ref_lse).max() <= (1e-5 if tol == TOL_F32 else 1e-2)
    return got


NESTED_CASES = [
    # (case, chain length, visibility or None = branch g sees g/gamma of the chain)
    (W.AttnCase("nested_f32", (77, 0, 130), 3, 5, 6, 2, 128, "f32", "f32", "f32", "f32", seed=11), 10, None),
    (W.AttnCase("nested_f32_paged_long_chain", (300, 45), 4, 9, 8, 2, 64, "f32", "f32", "f32", "f32", paged=True,
                seed=12), 150, None),
    # Algorithm 1's shape: gamma steps of L tokens, step j conditioned on steps 0..j-1, so C = (gamma-1)*L
    (W.AttnCase("nested_bf16_steps", (1000,), 4, 20, 16, 2, 128, seed=13), 60, None),
    # chain longer than a key tile, visibility neither monotone nor the same in the two requests, one branch
    # sees nothing and one everything; row tiles straddle branches (L*G = 210)
    (W.AttnCase("nested_bf16_ragged_vis", (130, 515), 4, 70, 6, 2, 128, paged=True, seed=14), 150,
     [[150, 0, 67, 64], [1, 149, 0, 3]]),
    (W.AttnCase("nested_fp8", (900,), 3, 33, 10, 2, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16", seed=15), 70, None),
    (W.AttnCase("nested_fp8_bf16_branch", (515, 64), 2, 40, 8, 1, 128, "bf16", "fp8_e4m3", "bf16", "f32", paged=True,
                seed=16), 90, [[90, 13], [0, 64]]),
    # no prefix at all: the chain and the branch are all there is; the first branch sees only itself
    (W.AttnCase("nested_bf16_no_prefix", (0,), 3, 8, 8, 2, 128, seed=17), 16, None),
    (W.AttnCase("nested_bf16_single_token_branches", (321,), 8, 1, 40, 8, 128, seed=18), 7, None),
]


@pytest.mark.parametrize("case,chain_len,vis", NESTED_CASES, ids=lambda x: getattr(x, "name", None))
def test_nested_small_cases(oracle, case, chain_len, vis):
    tol = TOL_F32 if case.kv_dtype == "f32" else TOL_LOWP
    for split in ((0,) if case.kv_dtype == "f32" else (0, 64, 256)):
        check_nested(oracle, case, chain_len, tol, None if vis is None else np.array(vis), split)


@pytest.mark.parametrize("shape", [0, 1])
def test_nested_every_kernel_shape(oracle, shape, monkeypatch):
    monkeypatch.setattr("gpu_util.KERNEL_SHAPE", shape + 1)
    for case, chain_len, vis in (NESTED_CASES[2], NESTED_CASES[3], NESTED_CASES[4]):
        for split in (0, 192):
            check_nested(oracle, case, chain_len, TOL_LOWP, None if vis is None else np.array(vis), split)


@pytest.mark.parametrize("shape", [1, 2])
@pytest.mark.parametrize("case", [NESTED_CASES[0][0], NESTED_CASES[3][0]], ids=lambda c: c.name)
def test_nested_with_nothing_visible_is_the_flat_call_bit_for_bit(case, shape, monkeypatch):
    """A chain no branch sees (all of chain_vis zero), and an empty chain, must reproduce la_verify_attention
    exactly when both run the same kernel shape (the flat call alone may also choose a streaming shape): no tile of
    the chain is touched."""
    from gpu_util import run_attention, run_attention_nested
    if case.kv_dtype != "f32":
        monkeypatch.setattr("gpu_util.KERNEL_SHAPE", shape)
    elif shape != 1:
        pytest.skip("one fp32 kernel")
    inp = W.make_attention_inputs(case)
    flat, flat_lse = run_attention(case, inp)
    chain = W.make_chain_inputs(case, 40, inp, np.zeros((case.B, case.gamma), dtype=np.int32))
    got, lse = run_attention_nested(case, inp, chain)
    assert np.array_equal(got, flat) and np.array_equal(lse, flat_lse)
    empty = W.make_chain_inputs(case, 0, inp)
    got, lse = run_attention_nested(case, inp, empty)
    assert np.array_equal(got, flat) and np.array_equal(lse, flat_lse)


def test_nested_rejects_bad_visibility():
    from gpu_util import run_attention_nested
    from paper_2506_19830_amd import binding as B
    case = NESTED_CASES[0][0]
    inp = W.make_attention_inputs(case)
    for bad in (11, -1):
        vis = np.zeros((case.B, case.gamma), dtype=np.int32)
        vis[1, 2] = bad
        with pytest.raises(B.LaError):
            run_attention_nested(case, inp, W.make_chain_inputs(case, 10, inp, vis))


# ----------------------------------------------------------------------------------------- draft trees

def check_tree(oracle, case, width, depth, step_len, tol, kv_split_tokens=0, edit=None):
    from gpu_util import row_errors, run_attention_tree
    inp = W.make_attention_inputs(case)
    tree = W.make_tree_inputs(case, width, depth, step_len, inp)
    if edit is not None:
        edit(tree)
    print(f"tree case {case.name} prefix={case.prefix_lens} gamma={case.gamma} L={case.L} W={width} depth={depth} "
          f"step={step_len} masks={[[hex(int(m)) for m in row] for row in tree['seg_mask']]} kv={case.kv_dtype} "
          f"br={case.branch_kv_dtype} split={kv_split_tokens}", flush=True)
    got, lse = run_attention_tree(case, inp, tree, kv_split_tokens)
    ref, ref_lse = oracle.verify_attention(**inp, **tree, q_dtype=case.q_dtype, kv_dtype=case.kv_dtype,
                                           branch_kv_dtype=case.branch_kv_dtype, block_size=case.block_size,
                                           scale=case.scale)
    assert np.isfinite(got).all()
    err = row_errors(got, ref)
    assert err.max() <= tol, f"max row error {err.max():.3e} at row {err.argmax()}"
    assert np.abs(lse - ref_lse).max() <= (1e-5 if tol == TOL_F32 else 1e-2)
    return got


def high_segments(tree):
    """Move the segment ids to the top of the 64-bit mask (ids 63, 62, ...): the upper mask word is exercised."""
    n = int(tree["pool_seg"].max()) + 1
    tree["pool_seg"][:] = 63 - tree["pool_seg"]
    tree["seg_mask"][:] = [[sum(1 << (63 - s) for s in range(n) if (int(m) >> s) & 1) for m in row]
                           for row in tree["seg_mask"]]


TREE_CASES = [
    # (case, width, depth, tokens per step, edit)
    (W.AttnCase("tree_f32", (77, 0, 130), 5, 5, 6, 2, 128, "f32", "f32", "f32", "f32", seed=51), 2, 3, 7, None),
    (W.AttnCase("tree_f32_no_prefix_high_ids", (0, 3), 4, 9, 8, 2, 64, "f32", "f32", "f32", "f32", paged=True,
                seed=52), 3, 2, 30, high_segments),
    # W = 2, three positions: 14 nodes of 20 tokens = 280 pool tokens (more than four key tiles, ragged tail)
    (W.AttnCase("tree_bf16_w2", (1000,), 6, 20, 16, 2, 128, seed=53), 2, 3, 20, None),
    # row tiles straddle branches (L*G = 210); W = 3, two positions: 12 nodes
    (W.AttnCase("tree_bf16_w3_paged", (130, 515), 5, 70, 6, 2, 128, paged=True, seed=54), 3, 2, 11, high_segments),
    (W.AttnCase("tree_fp8", (900,), 4, 33, 10, 2, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16", seed=55), 2, 4, 9,
     None),
    (W.AttnCase("tree_fp8_bf16_branch", (515, 64), 3, 40, 8, 1, 128, "bf16", "fp8_e4m3", "bf16", "f32", paged=True,
                seed=56), 2, 2, 40, None),
    (W.AttnCase("tree_bf16_no_prefix", (0,), 4, 8, 8, 2, 128, seed=57), 2, 2, 5, None),
    # 62 nodes of 3 tokens: nearly every bit of the mask in use
    (W.AttnCase("tree_bf16_62_nodes", (321,), 8, 1, 40, 8, 128, seed=58), 2, 5, 3, None),
]


@pytest.mark.parametrize("case,width,depth,step_len,edit", TREE_CASES, ids=lambda x: getattr(x, "name", None))
def test_tree_small_cases(oracle, case, width, depth, step_len, edit):
    tol = TOL_F32 if case.kv_dtype == "f32" else TOL_LOWP
    for split in ((0,) if case.kv_dtype == "f32" else (0, 64, 256)):
        check_tree(oracle, case, width, depth, step_len, tol, split, edit)


@pytest.mark.parametrize("shape", [0, 1])
def test_tree_every_kernel_shape(oracle, shape, monkeypatch):
    monkeypatch.setattr("gpu_util.KERNEL_SHAPE", shape + 1)
    for case, width, depth, step_len, edit in (TREE_CASES[2], TREE_CASES[3], TREE_CASES[4]):
        for split in (0, 192):
            check_tree(oracle, case, width, depth, step_len, TOL_LOWP, split, edit)


def test_tree_whose_masks_are_leading_parts_equals_the_nested_call():
    """The same visibility said in both vocabularies: the two entry points must agree bit for bit."""
    from gpu_util import run_attention_nested, run_attention_tree
    case = W.AttnCase("tree_chain", (300, 70), 4, 12, 8, 2, 128, seed=59)
    inp = W.make_attention_inputs(case)
    tree = W.make_tree_inputs(case, 1, 6, 25, inp)                 # a chain of 6 steps of 25 tokens
    tree["seg_mask"][:] = [[0, 0b1, 0b111, 0b111111], [0b11, 0, 0b1111, 0b11111]]
    vis = np.array([[0, 25, 75, 150], [50, 0, 100, 125]], dtype=np.int32)
    a, la = run_attention_tree(case, inp, tree)
    b, lb = run_attention_nested(case, inp, {"k_chain": tree["k_pool"], "v_chain": tree["v_pool"], "chain_vis": vis})
    assert np.array_equal(a, b) and np.array_equal(la, lb)


def test_tree_with_empty_masks_is_the_flat_call(monkeypatch):
    """MFMA path: pool tiles nobody sees are skipped, so the result is the flat call's bit for bit when both run the
    same kernel shape (the flat call alone may also choose a streaming shape).  fp32 path: the unseen tokens are
    walked with weight zero, which regroups the 64-key steps of the running softmax: equal up to fp32 rounding."""
    from gpu_util import row_errors, run_attention, run_attention_tree
    for case in (TREE_CASES[0][0], TREE_CASES[2][0]):
        monkeypatch.setattr("gpu_util.KERNEL_SHAPE", 0 if case.kv_dtype == "f32" else 2)
        inp = W.make_attention_inputs(case)
        flat, flat_lse = run_attention(case, inp)
        tree = W.make_tree_inputs(case, 2, 2, 10, inp)
        tree["seg_mask"][:] = 0
        got, lse = run_attention_tree(case, inp, tree)
        if case.kv_dtype == "f32":
            assert row_errors(got, flat).max() < 1e-6 and np.abs(lse - flat_lse).max() < 1e-6
        else:
            assert np.array_equal(got, flat) and np.array_equal(lse, flat_lse)


def test_tree_rejects_bad_segments():
    from gpu_util import run_attention_tree
    from paper_2506_19830_amd import binding as B
    case = TREE_CASES[0][0]
    inp = W.make_attention_inputs(case)
    for bad in (64, -1):
        tree = W.make_tree_inputs(case, 2, 2, 4, inp)
        tree["pool_seg"][1, 3] = bad
        with pytest.raises(B.LaError):
            run_attention_tree(case, inp, tree)


def test_mfma_fp32_output_is_tight(oracle):
    """With fp32 output the low-precision steps left are P rounded to bf16 and Q rounded to bf16 again after the
    score scale is folded in: errors stay at a few 1e-3, well inside the 2e-2 bar."""
    case = replace(MFMA_CASES[0], out_dtype="f32")
    from gpu_util import row_errors, run_attention
    inp = W.make_attention_inputs(case)
    got, _ = run_attention(case, inp, 256)
    ref, _ = oracle_attention(oracle, case, inp)
    assert row_errors(got, ref).max() < 1e-2


def test_split_count_changes_nothing_beyond_rounding(oracle):
    from gpu_util import row_errors, run_attention
    case = replace(MFMA_CASES[0], out_dtype="f32")
    inp = W.make_attention_inputs(case)
    a, _ = run_attention(case, inp, 64)
    b, _ = run_attention(case, inp, 1024)
    assert row_errors(a, b).max() < 1.5e-2    # each run is within ~5e-3 of the exact result (P, Q*scale in bf16)


def test_deterministic_and_block_permutation_invariant():
    from gpu_util import run_attention
    case = MFMA_CASES[2]
    inp = W.make_attention_inputs(case)
    a, la_ = run_attention(case, inp, 256)
    b, lb = run_attention(case, inp, 256)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(la_, lb)
    nb = inp["k_cache"].shape[0]
    perm = np.random.default_rng(0).permutation(nb)
    moved = dict(inp)
    moved["k_cache"] = np.empty_like(inp["k_cache"])
    moved["v_cache"] = np.empty_like(inp["v_cache"])
    moved["k_cache"][perm] = inp["k_cache"]
    moved["v_cache"][perm] = inp["v_cache"]
    moved["block_tables"] = perm[inp["block_tables"]].astype(np.int32)
    c, _ = run_attention(case, moved, 256)
    np.testing.assert_array_equal(a, c)


def test_branch_isolation_and_causality_on_gpu():
    from gpu_util import run_attention
    case = MFMA_CASES[1]
    inp = W.make_attention_inputs(case)
    base, _ = run_attention(case, inp, 64)
    pert = {k: (None if v is None else v.copy()) for k, v in inp.items()}
    pert["k_branch"][:, 0] ^= 0x0040          # flip a mantissa bit of every K of branch 0
    pert["v_branch"][:, 2] ^= 0x0040
    out, _ = run_attention(case, pert, 64)
    np.testing.assert_array_equal(out[:, 1], base[:, 1])
    np.testing.assert_array_equal(out[:, 3], base[:, 3])
    assert not np.array_equal(out[:, 0], base[:, 0]) and not np.array_equal(out[:, 2], base[:, 2])
    pert = {k: (None if v is None else v.copy()) for k, v in inp.items()}
    pert["k_branch"][:, :, 40:] ^= 0x0040     # tokens after 39 are invisible to rows 0..39
    pert["v_branch"][:, :, 40:] ^= 0x0040
    out, _ = run_attention(case, pert, 64)
    np.testing.assert_array_equal(out[:, :, :40], base[:, :, :40])
    assert not np.array_equal(out[:, :, 40], base[:, :, 40])


def test_fp8_scale_identities_on_gpu():
    from gpu_util import row_errors, run_attention
    case = replace(MFMA_CASES[3], out_dtype="f32")
    inp = W.make_attention_inputs(case)
    base, _ = run_attention(case, inp, 256)
    twice = dict(inp)
    twice["v_scale"] = inp["v_scale"] * np.float32(2.0)
    out, _ = run_attention(case, twice, 256)
    np.testing.assert_array_equal(out, 2.0 * base)
    shifted = dict(inp)
    shifted["k_scale"] = inp["k_scale"] * np.float32(4.0)
    out, _ = run_attention(case, shifted, 256, scale=case.scale / 4.0)
    assert row_errors(out, base).max() < 1e-5


# ----------------------------------------------------------------------------------------- benchmark configurations

def test_config2_full(oracle):
    case, _ = W.config(2)
    check_full(oracle, case, TOL_LOWP)


def sampled_rows(case, n_random, seed=0):
    """First and last token of every branch for every head, plus random rows."""
    ids = []
    for b in range(case.B):
        for g in range(case.gamma):
            for i in (0, case.L - 1):
                for h in range(case.Hq):
                    ids.append(((b * case.gamma + g) * case.L + i) * case.Hq + h)
    total = case.B * case.gamma * case.L * case.Hq
    ids.extend(np.random.default_rng(seed).integers(0, total, size=n_random).tolist())
    return np.unique(np.asarray(ids, dtype=np.int64))


@pytest.mark.parametrize("n", [3, 4])
def test_full_size_configs_every_row(oracle, n):
    """Configurations 3 and 4 at full size, in the launch configuration the benchmark uses, every output row against
    the oracle (configuration 4: about a teraflop of fp64 on the host cores)."""
    case, _ = W.config(n)
    check_full(oracle, case, TOL_LOWP)


@pytest.mark.parametrize("n", [3, 4, 5])
def test_full_size_configs_on_sampled_rows(oracle, n):
    """Configurations 3-5 at full size in the launch configuration the benchmark uses (automatic split); the
    oracle evaluates first/last token of every branch and head plus random rows (config 5: one layer)."""
    from gpu_util import row_errors, run_attention
    case, _ = W.config(n)
    print(f"config {n}: {case.name}", flush=True)
    inp = W.make_attention_inputs(case)
    got, lse = run_attention(case, inp)
    assert np.isfinite(got).all()
    ids = sampled_rows(case, 600)
    ref, ref_lse = oracle_attention(oracle, case, inp, row_ids=ids)
    err = row_errors(got.reshape(-1, case.D)[ids], ref)
    assert err.max() <= TOL_LOWP, f"max row error {err.max():.3e}"
    assert np.abs(lse.reshape(-1)[ids] - ref_lse).max() <= 1e-2


def test_very_long_ragged_paged_prefix_on_sampled_rows(oracle, monkeypatch):
    """A 300001-token paged fp8 prefix next to a short one, through both row-tile kernel shapes: automatic splits, the
    longest chunk the block ids a workgroup keeps in LDS allow (4072 blocks nominal, a few more once the tiles are
    dealt out evenly; 4096 slots), many short chunks (74 per request: the general merge form)."""
    from gpu_util import row_errors, run_attention
    case = W.AttnCase("long_prefix", (300001, 777), 2, 5, 8, 2, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16",
                      paged=True, seed=61)
    import torch
    dev = W.make_attention_inputs_device(case)
    inp = W.device_inputs_to_numpy(case, dev)
    ids = sampled_rows(case, 100)
    ref, ref_lse = oracle_attention(oracle, case, inp, row_ids=ids)
    for shape, split in ((0, 0), (1, 0), (0, 65152), (1, 4096)):
        monkeypatch.setattr("gpu_util.KERNEL_SHAPE", shape + 1)
        print(f"long prefix: shape {shape} split {split}", flush=True)
        got, lse = run_attention(case, inp, split, dev=dev)
        err = row_errors(got.reshape(-1, case.D)[ids], ref)
        print(f"long prefix: max row error {err.max():.3e}", flush=True)
        # the roundings of the path (Q times the score scale to bf16 a second time, P to bf16, the output to bf16) are
        # per element and do not accumulate with the prefix length: at 300001 tokens the error must still leave 40 %
        # of the 2e-2 bound unused
        assert err.max() <= 1.2e-2, f"max row error {err.max():.3e}"
        assert np.abs(lse.reshape(-1)[ids] - ref_lse).max() <= 1e-2
    # a chunk longer than the block ids a workgroup can hold is refused when it is asked for explicitly
    from paper_2506_19830_amd import binding as B
    with pytest.raises(B.LaError):
        run_attention(case, inp, 65536, dev=dev)
    del dev
    torch.cuda.empty_cache()


# ----------------------------------------------------------------------------------------- random shapes

def random_case(rng, idx):
    """A small random problem: every structural parameter drawn, sizes kept to what the oracle does in a second."""
    dt = [("bf16", "bf16", "bf16", "bf16"), ("bf16", "fp8_e4m3", "fp8_e4m3", "bf16"),
          ("bf16", "fp8_e4m3", "bf16", "f32"), ("bf16", "bf16", "bf16", "f32"), ("f32", "f32", "f32", "f32")][idx % 5]
    hkv = int(rng.choice([1, 2, 4, 8]))
    g = int(rng.choice([1, 2, 5, 8, 16]))
    nreq = int(rng.choice([1, 2, 3, 6]))
    gamma = int(rng.choice([1, 2, 3, 5, 8]))
    L = int(rng.choice([1, 2, 7, 16, 33, 64, 90]))
    while nreq * gamma * L * hkv * g > 6000:          # rows; keeps the oracle quick
        L = max(1, L // 2)
    bs = int(rng.choice([16, 32, 64, 128]))
    prefix = tuple(int(x) for x in rng.choice([0, 1, 15, 64, 65, 200, 513, 1100, 2500], size=nreq))
    D = 128 if dt[0] != "f32" else int(rng.choice([64, 128, 256]))
    return W.AttnCase(f"rand{idx}", prefix, gamma, L, hkv * g, hkv, D, *dt, block_size=bs,
                      paged=bool(rng.integers(0, 2)), seed=100 + idx)


@pytest.mark.parametrize("idx", range(30))
def test_random_shapes(oracle, idx):
    """Flat, nested and tree calls on randomly drawn shapes (heads, group size, requests, branches, branch length,
    block size, ragged prefixes, paging, dtypes, split), each against the oracle."""
    rng = np.random.default_rng(1000 + idx)
    case = random_case(rng, idx)
    tol = TOL_F32 if case.kv_dtype == "f32" else TOL_LOWP
    split = 0 if case.kv_dtype == "f32" else int(rng.choice([0, 64, 128, 448]))
    kind = idx % 3
    if kind == 0:
        check_full(oracle, case, tol, kv_split_tokens=split)
    elif kind == 1:
        C = int(rng.choice([1, 5, 64, 65, 130]))
        vis = rng.integers(0, C + 1, size=(case.B, case.gamma))
        check_nested(oracle, case, C, tol, vis, split)
    else:
        width, depth = [(1, 4), (2, 2), (2, 3), (3, 2), (4, 2)][int(rng.integers(0, 5))]
        check_tree(oracle, case, width, depth, int(rng.choice([1, 4, 17, 40])), tol, split)
