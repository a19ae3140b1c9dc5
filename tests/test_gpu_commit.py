"""GPU parity of la_kv_commit against the CPU oracle, through the C ABI.  Byte work: every comparison is exact."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from paper_2506_19830_amd import binding as B
from paper_2506_19830_amd import workloads as W

pytestmark = pytest.mark.gpu


def oracle_commit(oracle, case, inp, chain, dec):
    return oracle.kv_commit(inp["k_cache"], inp["v_cache"], inp["block_tables"], inp["prefix_lens"], inp["k_branch"],
                            inp["v_branch"], None if chain is None else chain["k_chain"],
                            None if chain is None else chain["v_chain"], dec["src_branch"], dec["n_chain"],
                            dec["n_own"], inp["k_scale"], inp["v_scale"], kv_dtype=case.kv_dtype,
                            branch_kv_dtype=case.branch_kv_dtype, block_size=case.block_size)


def gpu_commit(case, inp, chain, dec):
    """One layer.  Returns (k_cache bits, v_cache bits, new_prefix_lens) as numpy."""
    from gpu_util import attn_desc, upload_attention
    dev = upload_attention(case, inp)
    kch = vch = None
    if chain is not None and chain["k_chain"].shape[1] > 0:
        kch = B.to_device(chain["k_chain"], case.branch_kv_dtype)
        vch = B.to_device(chain["v_chain"], case.branch_kv_dtype)
    d = {k: torch.from_numpy(v).cuda() for k, v in dec.items()}
    new_lens = torch.full((case.B,), -7, dtype=torch.int32, device="cuda")
    B.la_kv_commit(attn_desc(case), dev["k_cache"], dev["v_cache"], dev["block_tables"], dev["prefix_lens"],
                   [int(x) for x in inp["prefix_lens"]], dev["k_branch"], dev["v_branch"], kch, vch, d["src_branch"],
                   d["n_chain"], d["n_own"], dev["k_scale"], dev["v_scale"], new_lens)
    torch.cuda.synchronize()
    return (W.device_bits(dev["k_cache"], case.kv_dtype), W.device_bits(dev["v_cache"], case.kv_dtype),
            new_lens.cpu().numpy())


CASES = [
    (W.AttnCase("commit_f32_paged", (37, 0, 130), 3, 9, 4, 2, 64, "f32", "f32", "f32", "f32", paged=True, seed=31,
                spare_tokens=40), 25),
    (W.AttnCase("commit_bf16", (100, 15), 4, 20, 4, 2, 128, seed=32, spare_tokens=64), 30),
    (W.AttnCase("commit_bf16_d256_block64", (300,), 2, 70, 2, 1, 256, seed=33, block_size=64, paged=True,
                spare_tokens=200), 130),
    (W.AttnCase("commit_fp8_fp8", (77, 1000), 2, 5, 16, 8, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16", paged=True,
                seed=34, spare_tokens=24), 12),
    (W.AttnCase("commit_fp8_from_bf16", (50, 9, 0), 3, 33, 8, 4, 128, "bf16", "fp8_e4m3", "bf16", "bf16", paged=True,
                seed=35, spare_tokens=100), 60),
]


@pytest.mark.parametrize("case,C", CASES, ids=lambda x: getattr(x, "name", None))
def test_commit_matches_the_oracle_byte_for_byte(oracle, case, C):
    inp = W.make_attention_inputs(case)
    chain = W.make_chain_inputs(case, C, inp)
    B_ = case.B
    full = (np.full(B_, case.gamma - 1), np.full(B_, C), np.full(B_, case.L))
    none = (np.zeros(B_, dtype=np.int32),) * 3
    for decisions in (None, full, none):
        dec = W.make_commit_inputs(case, C, decisions)
        print(f"commit case {case.name} C={C} decisions={ {k: v.tolist() for k, v in dec.items()} }", flush=True)
        kc, vc, new_lens = gpu_commit(case, inp, chain, dec)
        rk, rv, rl = oracle_commit(oracle, case, inp, chain, dec)
        assert np.array_equal(new_lens, rl)
        assert np.array_equal(kc, rk)
        assert np.array_equal(vc, rv)


def test_commit_without_a_chain(oracle):
    case, _ = CASES[1]
    inp = W.make_attention_inputs(case)
    dec = W.make_commit_inputs(case, 0)
    kc, vc, new_lens = gpu_commit(case, inp, None, dec)
    rk, rv, rl = oracle_commit(oracle, case, inp, None, dec)
    assert np.array_equal(new_lens, rl) and np.array_equal(kc, rk) and np.array_equal(vc, rv)


def test_quantiser_on_every_rounding_boundary(oracle):
    """A bf16 source placed on and around every midpoint between neighbouring e4m3 values (all of them are exact in
    bf16 or get rounded to a neighbour, both fine: the oracle sees the same bits), saturating values and signed
    zeros, through a scale of one and an awkward one."""
    codes = np.arange(127, dtype=np.uint8)
    vals = oracle.widen(codes, "fp8_e4m3")
    mids = (vals[:-1] + vals[1:]) / 2
    pts = np.concatenate([vals, mids, mids * (1 + 2.0 ** -7), mids * (1 - 2.0 ** -7), [449, 460, 464, 480, 1e4, 1e30]])
    pts = np.concatenate([pts, -pts]).astype(np.float32)
    D, Hkv = 128, 2
    L = -(-pts.size // (D * Hkv))
    case = W.AttnCase("commit_boundaries", (16,), 1, L, 2, Hkv, D, "bf16", "fp8_e4m3", "bf16", "bf16", seed=36,
                      spare_tokens=L)
    inp = W.make_attention_inputs(case)
    for scales in ((1.0, 1.0), (0.37, 3.3)):
        sc = np.array(scales, dtype=np.float32)
        inp["k_scale"], inp["v_scale"] = sc, sc[::-1].copy()
        src = np.zeros(L * Hkv * D, dtype=np.float32)
        src[:pts.size] = pts
        src = src.reshape(1, 1, L, Hkv, D)
        inp["k_branch"] = W.encode_bf16(src * inp["k_scale"][None, None, None, :, None])   # quotient lands near pts
        inp["v_branch"] = W.encode_bf16(src * inp["v_scale"][None, None, None, :, None])
        dec = W.make_commit_inputs(case, 0, ([0], [0], [L]))
        kc, vc, _ = gpu_commit(case, inp, None, dec)
        rk, rv, _ = oracle_commit(oracle, case, inp, None, dec)
        assert np.array_equal(kc, rk) and np.array_equal(vc, rv)


def test_commit_of_many_layers_in_one_call(oracle):
    """Layers back to back in one allocation, per-layer scales: one launch must equal the oracle layer by layer."""
    from gpu_util import attn_desc
    case = W.AttnCase("commit_layers", (90, 33), 3, 12, 8, 4, 128, "bf16", "fp8_e4m3", "bf16", "bf16", paged=True,
                      seed=37, spare_tokens=40)
    C, NL = 20, 5
    per_layer = [W.make_attention_inputs(W.with_layer(case, l)) for l in range(NL)]
    chains = [W.make_chain_inputs(W.with_layer(case, l), C, per_layer[l]) for l in range(NL)]
    tables = per_layer[0]["block_tables"]          # one block table for all layers, as in a real cache
    for x in per_layer:
        x["block_tables"] = tables
    dec = W.make_commit_inputs(case, C)

    def stack(key, dtype, src=per_layer):
        return torch.stack([B.to_device(x[key], dtype) for x in src]).contiguous()

    kc, vc = stack("k_cache", case.kv_dtype), stack("v_cache", case.kv_dtype)
    kb, vb = stack("k_branch", case.branch_kv_dtype), stack("v_branch", case.branch_kv_dtype)
    kch, vch = stack("k_chain", case.branch_kv_dtype, chains), stack("v_chain", case.branch_kv_dtype, chains)
    ks = torch.stack([torch.from_numpy(x["k_scale"]) for x in per_layer]).cuda()
    vs = torch.stack([torch.from_numpy(x["v_scale"]) for x in per_layer]).cuda()
    layers = B.la_layer_strides(num_layers=NL, cache_stride=kc[0].numel(), branch_stride=kb[0].numel(),
                                chain_stride=kch[0].numel(), scale_stride=case.Hkv)
    d = {k: torch.from_numpy(v).cuda() for k, v in dec.items()}
    new_lens = torch.full((case.B,), -7, dtype=torch.int32, device="cuda")
    B.la_kv_commit(attn_desc(case), kc, vc, torch.from_numpy(tables).cuda(),
                   torch.from_numpy(per_layer[0]["prefix_lens"]).cuda(), [int(x) for x in case.prefix_lens], kb, vb,
                   kch, vch, d["src_branch"], d["n_chain"], d["n_own"], ks, vs, new_lens, layers)
    torch.cuda.synchronize()
    for l in range(NL):
        rk, rv, rl = oracle_commit(oracle, case, per_layer[l], chains[l], dec)
        assert np.array_equal(W.device_bits(kc[l], case.kv_dtype), rk), l
        assert np.array_equal(W.device_bits(vc[l], case.kv_dtype), rv), l
        assert np.array_equal(new_lens.cpu().numpy(), rl)


def test_commit_then_verify_equals_the_nested_pass(oracle):
    """The use the commit is for: after it, a flat verification over the grown prefix must agree with the oracle's
    attention over the oracle's committed cache (bf16 tolerance), i.e. the two entry points compose."""
    from gpu_util import attn_desc, row_errors, run_attention, upload_attention
    case = W.AttnCase("commit_then_verify", (500,), 4, 16, 8, 2, 128, seed=38, spare_tokens=64)
    C = 48
    inp = W.make_attention_inputs(case)
    chain = W.make_chain_inputs(case, C, inp)
    dec = W.make_commit_inputs(case, C, ([2], [32], [16]))
    dev = upload_attention(case, inp)
    d = {k: torch.from_numpy(v).cuda() for k, v in dec.items()}
    new_lens = torch.zeros((case.B,), dtype=torch.int32, device="cuda")
    B.la_kv_commit(attn_desc(case), dev["k_cache"], dev["v_cache"], None, dev["prefix_lens"], [500],
                   dev["k_branch"], dev["v_branch"], B.to_device(chain["k_chain"], "bf16"),
                   B.to_device(chain["v_chain"], "bf16"), d["src_branch"], d["n_chain"], d["n_own"], None, None,
                   new_lens)
    torch.cuda.synchronize()
    grown = replace(case, prefix_lens=(548,), spare_tokens=16)      # same max_blocks: ceil(564/16) = ceil(564/16)
    assert grown.max_blocks == case.max_blocks
    dev["prefix_lens"] = new_lens
    inp2 = dict(inp, prefix_lens=np.array([548], dtype=np.int32))
    got, _ = run_attention(grown, inp2, dev=dev)
    rk, rv, rl = oracle_commit(oracle, case, inp, chain, dec)
    assert rl.tolist() == [548]
    ref, _ = oracle.verify_attention(**dict(inp2, k_cache=rk, v_cache=rv), q_dtype="bf16", kv_dtype="bf16",
                                     branch_kv_dtype="bf16", block_size=16, scale=case.scale)
    assert row_errors(got, ref).max() <= 2e-2


def test_device_side_clamps_keep_the_writes_inside_the_table(oracle):
    """Decisions outside their ranges (they come from another kernel, the host never sees them) are clamped:
    the result equals the oracle's for the clamped decisions and nothing else is written."""
    case, C = CASES[1]
    inp = W.make_attention_inputs(case)
    chain = W.make_chain_inputs(case, C, inp)
    wild = W.make_commit_inputs(case, C, ([case.gamma + 3, -2], [C + 50, -1], [case.L + 9, 5]))
    tame = W.make_commit_inputs(case, C, ([case.gamma - 1, 0], [C, 0], [case.L, 5]))
    kc, vc, new_lens = gpu_commit(case, inp, chain, wild)
    rk, rv, rl = oracle_commit(oracle, case, inp, chain, tame)
    assert np.array_equal(new_lens, rl) and np.array_equal(kc, rk) and np.array_equal(vc, rv)


# ------------------------------------------------------------------------------------------ draft trees

def labelled_tree(case, inp, width, depth, step_len, seed):
    """The generators' tree pool with the node labels shuffled inside each request (interleaved nodes, different per
    request) and the highest node relabelled 63, so that the whole 64-bit mask is exercised."""
    tree = W.make_tree_inputs(case, width, depth, step_len, inp)
    rng = np.random.default_rng(seed)
    seg = tree["pool_seg"].copy()
    top = int(seg.max())
    for b in range(case.B):
        rng.shuffle(seg[b])
        seg[b] = np.where(seg[b] == top, 63, seg[b])
    return dict(tree, pool_seg=seg), top


def random_masks(rng, B_, top, p):
    """Each node 0..top-1 and node 63 accepted with probability p."""
    bits = rng.random((B_, top + 1)) < p
    m = np.zeros(B_, dtype=np.uint64)
    for b in range(B_):
        for n in range(top):
            if bits[b, n]:
                m[b] |= np.uint64(1) << np.uint64(n)
        if bits[b, top]:
            m[b] |= np.uint64(1) << np.uint64(63)
    return m


def oracle_commit_tree(oracle, case, inp, tree, cm, src, nown):
    return oracle.kv_commit_tree(inp["k_cache"], inp["v_cache"], inp["block_tables"], inp["prefix_lens"],
                                 inp["k_branch"], inp["v_branch"], tree["k_pool"], tree["v_pool"], tree["pool_seg"],
                                 cm, src, nown, inp["k_scale"], inp["v_scale"], kv_dtype=case.kv_dtype,
                                 branch_kv_dtype=case.branch_kv_dtype, block_size=case.block_size)


def gpu_commit_tree(case, inp, tree, cm, src, nown):
    from gpu_util import attn_desc, upload_attention
    dev = upload_attention(case, inp)
    kp = B.to_device(tree["k_pool"], case.branch_kv_dtype)
    vp = B.to_device(tree["v_pool"], case.branch_kv_dtype)
    seg = torch.from_numpy(tree["pool_seg"]).cuda()
    mask = torch.from_numpy(np.asarray(cm, dtype=np.uint64).view(np.int64)).cuda()
    src_d = torch.from_numpy(np.asarray(src, dtype=np.int32)).cuda()
    nown_d = torch.from_numpy(np.asarray(nown, dtype=np.int32)).cuda()
    new_lens = torch.full((case.B,), -7, dtype=torch.int32, device="cuda")
    B.la_kv_commit_tree(attn_desc(case), dev["k_cache"], dev["v_cache"], dev["block_tables"], dev["prefix_lens"],
                        [int(x) for x in inp["prefix_lens"]], dev["k_branch"], dev["v_branch"], kp, vp, seg, mask,
                        src_d, nown_d, dev["k_scale"], dev["v_scale"], new_lens)
    torch.cuda.synchronize()
    return (W.device_bits(dev["k_cache"], case.kv_dtype), W.device_bits(dev["v_cache"], case.kv_dtype),
            new_lens.cpu().numpy())


# (case, width, depth, step_len): pools of 24 .. 320 tokens, i.e. from one to many workgroups per request
TREE_COMMIT_CASES = [
    (W.AttnCase("tree_commit_f32_paged", (37, 0, 130), 3, 9, 4, 2, 64, "f32", "f32", "f32", "f32", paged=True,
                seed=41, spare_tokens=9 + 24), 2, 2, 4),
    (W.AttnCase("tree_commit_bf16", (100, 15), 4, 20, 4, 2, 128, seed=42, spare_tokens=20 + 210), 2, 4, 7),
    (W.AttnCase("tree_commit_bf16_d256_block64", (300,), 2, 70, 2, 1, 256, seed=43, block_size=64, paged=True,
                spare_tokens=70 + 195), 3, 3, 5),
    (W.AttnCase("tree_commit_fp8_fp8", (77, 1000), 2, 5, 16, 8, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16",
                paged=True, seed=44, spare_tokens=5 + 320), 4, 2, 16),
    (W.AttnCase("tree_commit_fp8_from_bf16", (50, 9, 0), 3, 33, 8, 4, 128, "bf16", "fp8_e4m3", "bf16", "bf16",
                paged=True, seed=45, spare_tokens=33 + 186), 2, 5, 3),
    # one 16-byte piece per token: a workgroup spans 256 pool tokens
    (W.AttnCase("tree_commit_fp8_one_piece_per_token", (40, 3), 2, 300, 1, 1, 16, "bf16", "fp8_e4m3", "fp8_e4m3",
                "bf16", seed=46, spare_tokens=300 + 620), 2, 4, 20 + 0),
]


@pytest.mark.parametrize("case,width,depth,step_len", TREE_COMMIT_CASES, ids=lambda x: getattr(x, "name", None))
def test_tree_commit_matches_the_oracle_byte_for_byte(oracle, case, width, depth, step_len):
    inp = W.make_attention_inputs(case)
    tree, top = labelled_tree(case, inp, width, depth, step_len, case.seed)
    rng = np.random.default_rng(case.seed)
    for p in (0.5, 0.1, 1.0, 0.0):
        cm = random_masks(rng, case.B, top, p)
        src = rng.integers(0, case.gamma, size=case.B).astype(np.int32)
        nown = rng.integers(0, case.L + 1, size=case.B).astype(np.int32)
        print(f"tree commit case {case.name} p={p} masks={[hex(int(x)) for x in cm]} src={src.tolist()} "
              f"n_own={nown.tolist()}", flush=True)
        kc, vc, new_lens = gpu_commit_tree(case, inp, tree, cm, src, nown)
        rk, rv, rl = oracle_commit_tree(oracle, case, inp, tree, cm, src, nown)
        assert np.array_equal(new_lens, rl)
        assert np.array_equal(kc, rk)
        assert np.array_equal(vc, rv)


def test_tree_commit_with_an_empty_pool_appends_the_own_tokens_only(oracle):
    case = TREE_COMMIT_CASES[1][0]
    inp = W.make_attention_inputs(case)
    from gpu_util import attn_desc, upload_attention
    dev = upload_attention(case, inp)
    src, nown = np.array([3, 0], dtype=np.int32), np.array([20, 7], dtype=np.int32)
    new_lens = torch.full((case.B,), -7, dtype=torch.int32, device="cuda")
    B.la_kv_commit_tree(attn_desc(case), dev["k_cache"], dev["v_cache"], dev["block_tables"], dev["prefix_lens"],
                        [int(x) for x in inp["prefix_lens"]], dev["k_branch"], dev["v_branch"], None, None, None,
                        torch.full((case.B,), -1, dtype=torch.int64, device="cuda"), torch.from_numpy(src).cuda(),
                        torch.from_numpy(nown).cuda(), None, None, new_lens)
    torch.cuda.synchronize()
    rk, rv, rl = oracle_commit(oracle, case, inp, None, W.make_commit_inputs(case, 0, (src, [0, 0], nown)))
    assert np.array_equal(new_lens.cpu().numpy(), rl)
    assert np.array_equal(W.device_bits(dev["k_cache"], case.kv_dtype), rk)
    assert np.array_equal(W.device_bits(dev["v_cache"], case.kv_dtype), rv)


def test_tree_commit_clamps_and_ignores_labels_outside_the_mask_range(oracle):
    """Decisions outside their ranges are clamped as in the chain form; a pool token whose label is not in 0..63 is
    never kept (the oracle, which rejects such labels, is given the same pool with those tokens on a node that is
    not accepted)."""
    case, width, depth, step_len = TREE_COMMIT_CASES[1]
    inp = W.make_attention_inputs(case)
    tree, top = labelled_tree(case, inp, width, depth, step_len, 7)
    cm = np.array([0x8000000000000155, 0x2AA], dtype=np.uint64)              # request 0 leaves out node 1, request 1 node 0
    assert not (int(cm[0]) >> 1) & 1 and not (int(cm[1]) >> 0) & 1
    wild_seg = tree["pool_seg"].copy()
    wild_seg[0][wild_seg[0] == 1] = 64                                       # request 0: node 1's tokens, bad label
    wild_seg[1][wild_seg[1] == 0] = -3                                       # request 1: node 0's tokens, bad label
    kc, vc, new_lens = gpu_commit_tree(case, inp, dict(tree, pool_seg=wild_seg), cm, [case.gamma + 2, -1],
                                       [case.L + 5, 4])
    rk, rv, rl = oracle_commit_tree(oracle, case, inp, tree, cm, [case.gamma - 1, 0], [case.L, 4])
    assert np.array_equal(new_lens, rl) and np.array_equal(kc, rk) and np.array_equal(vc, rv)


def test_tree_commit_of_many_layers_in_one_call(oracle):
    from gpu_util import attn_desc
    case = W.AttnCase("tree_commit_layers", (90, 33), 3, 12, 8, 4, 128, "bf16", "fp8_e4m3", "bf16", "bf16", paged=True,
                      seed=47, spare_tokens=12 + 70)
    NL = 4
    per_layer = [W.make_attention_inputs(W.with_layer(case, l)) for l in range(NL)]
    trees = [labelled_tree(W.with_layer(case, l), per_layer[l], 2, 3, 5, 9)[0] for l in range(NL)]   # same labels
    tables = per_layer[0]["block_tables"]
    for x in per_layer:
        x["block_tables"] = tables
    rng = np.random.default_rng(9)
    cm = random_masks(rng, case.B, 13, 0.5)
    src, nown = np.array([2, 0], dtype=np.int32), np.array([12, 5], dtype=np.int32)

    def stack(key, dtype, src_list=per_layer):
        return torch.stack([B.to_device(x[key], dtype) for x in src_list]).contiguous()

    kc, vc = stack("k_cache", case.kv_dtype), stack("v_cache", case.kv_dtype)
    kb, vb = stack("k_branch", case.branch_kv_dtype), stack("v_branch", case.branch_kv_dtype)
    kp, vp = stack("k_pool", case.branch_kv_dtype, trees), stack("v_pool", case.branch_kv_dtype, trees)
    ks = torch.stack([torch.from_numpy(x["k_scale"]) for x in per_layer]).cuda()
    vs = torch.stack([torch.from_numpy(x["v_scale"]) for x in per_layer]).cuda()
    layers = B.la_layer_strides(num_layers=NL, cache_stride=kc[0].numel(), branch_stride=kb[0].numel(),
                                chain_stride=kp[0].numel(), scale_stride=case.Hkv)
    new_lens = torch.full((case.B,), -7, dtype=torch.int32, device="cuda")
    B.la_kv_commit_tree(attn_desc(case), kc, vc, torch.from_numpy(tables).cuda(),
                        torch.from_numpy(per_layer[0]["prefix_lens"]).cuda(), [int(x) for x in case.prefix_lens], kb,
                        vb, kp, vp, torch.from_numpy(trees[0]["pool_seg"]).cuda(),
                        torch.from_numpy(cm.view(np.int64)).cuda(), torch.from_numpy(src).cuda(),
                        torch.from_numpy(nown).cuda(), ks, vs, new_lens, layers)
    torch.cuda.synchronize()
    for l in range(NL):
        rk, rv, rl = oracle_commit_tree(oracle, case, per_layer[l], trees[l], cm, src, nown)
        assert np.array_equal(W.device_bits(kc[l], case.kv_dtype), rk), l
        assert np.array_equal(W.device_bits(vc[l], case.kv_dtype), rv), l
        assert np.array_equal(new_lens.cpu().numpy(), rl)


def test_select_commit_then_verify_on_a_tree(oracle):
    """The whole tree path: a tree verification pass, the walk over the verdicts (host), the tree commit, and a flat
    pass over the grown prefix; each stage against the oracle's."""
    from oracle import planner as P
    from gpu_util import attn_desc, row_errors, run_attention, run_attention_tree, upload_attention
    width, depth, step_len = 2, 3, 6
    parent = W.tree_parents(width, depth)
    nodes = parent.size                                                        # 14
    case = W.AttnCase("tree_cycle", (700, 45), nodes + 1, 10, 8, 2, 128, seed=48, spare_tokens=10 + nodes * step_len)
    inp = W.make_attention_inputs(case)
    tree = W.make_tree_inputs(case, width, depth, step_len, inp)
    # branch 0 continues the bare prefix, branch 1+n the path ending in node n
    masks = np.zeros((case.B, nodes + 1), dtype=np.uint64)
    for n in range(nodes):
        m, a = 0, n
        while a >= 0:
            m |= 1 << a
            a = int(parent[a])
        masks[:, 1 + n] = m
    tree = dict(tree, seg_mask=masks)
    got, _ = run_attention_tree(case, inp, tree)
    ref, _ = oracle.verify_attention(**inp, **tree, q_dtype="bf16", kv_dtype="bf16", branch_kv_dtype="bf16",
                                     block_size=case.block_size, scale=case.scale)
    assert row_errors(got, ref).max() <= 2e-2

    verdicts = np.zeros((case.B, nodes), dtype=bool)
    verdicts[0, [1, 4, 5, 11, 2]] = True             # request 0: node 1, then 4 (5 also matches), then 11 below 4
    verdicts[1, [3, 6]] = True                       # request 1: nothing at position 0 matches
    own_len = np.tile(np.arange(3, 3 + nodes + 1) % (case.L + 1), (case.B, 1)).astype(np.int32)
    d, cm, src, nown = B.la_step_select_tree(parent, verdicts, own_len)
    want = P.tree_output_construction(parent.tolist(), verdicts.tolist(), own_len.tolist())
    assert [tuple(int(x) for x in t) for t in zip(d, src, cm, nown)] == want
    assert d.tolist() == [3, 0] and src.tolist() == [12, 0]

    dev = upload_attention(case, inp)
    new_lens = torch.zeros((case.B,), dtype=torch.int32, device="cuda")
    B.la_kv_commit_tree(attn_desc(case), dev["k_cache"], dev["v_cache"], dev["block_tables"], dev["prefix_lens"],
                        [int(x) for x in inp["prefix_lens"]], dev["k_branch"], dev["v_branch"],
                        B.to_device(tree["k_pool"], "bf16"), B.to_device(tree["v_pool"], "bf16"),
                        torch.from_numpy(tree["pool_seg"]).cuda(), torch.from_numpy(cm.view(np.int64)).cuda(),
                        torch.from_numpy(src).cuda(), torch.from_numpy(nown).cuda(), None, None, new_lens)
    torch.cuda.synchronize()
    rk, rv, rl = oracle_commit_tree(oracle, case, inp, tree, cm, src, nown)
    assert np.array_equal(new_lens.cpu().numpy(), rl)
    assert rl.tolist() == [700 + 3 * step_len + int(nown[0]), 45 + int(nown[1])]
    assert np.array_equal(W.device_bits(dev["k_cache"], "bf16"), rk)

    grown = replace(case, prefix_lens=tuple(int(x) for x in rl), spare_tokens=0)
    if grown.max_blocks != case.max_blocks:          # keep the cache's shape: the table is the one already uploaded
        grown = replace(grown, spare_tokens=case.max_blocks * case.block_size - max(rl))
    assert grown.max_blocks == case.max_blocks
    dev["prefix_lens"] = new_lens
    inp2 = dict(inp, prefix_lens=rl)
    got2, _ = run_attention(grown, inp2, dev=dev)
    ref2, _ = oracle.verify_attention(**dict(inp2, k_cache=rk, v_cache=rv), q_dtype="bf16", kv_dtype="bf16",
                                      branch_kv_dtype="bf16", block_size=case.block_size, scale=case.scale)
    assert row_errors(got2, ref2).max() <= 2e-2
