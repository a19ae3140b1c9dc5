"""Helpers of the GPU parity tests: run the HIP library through its C ABI on numpy inputs from the seeded
generators and bring the results back as numpy.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from paper_2506_19830_amd import binding as B
from paper_2506_19830_amd import workloads as W


def upload_attention(case: W.AttnCase, inp: dict) -> dict:
    dev = {
        "q": B.to_device(inp["q"], case.q_dtype),
        "k_cache": B.to_device(inp["k_cache"], case.kv_dtype),
        "v_cache": B.to_device(inp["v_cache"], case.kv_dtype),
        "block_tables": None if inp["block_tables"] is None else torch.from_numpy(inp["block_tables"]).cuda(),
        "prefix_lens": torch.from_numpy(inp["prefix_lens"]).cuda(),
        "k_branch": B.to_device(inp["k_branch"], case.branch_kv_dtype),
        "v_branch": B.to_device(inp["v_branch"], case.branch_kv_dtype),
        "k_scale": None if inp["k_scale"] is None else torch.from_numpy(inp["k_scale"]).cuda(),
        "v_scale": None if inp["v_scale"] is None else torch.from_numpy(inp["v_scale"]).cuda(),
    }
    return dev


# kernel shape every descriptor built here asks for (0: the library chooses); tests that walk the shapes patch it
KERNEL_SHAPE = 0


def attn_desc(case: W.AttnCase, kv_split_tokens: int = 0, scale=None):
    return B.make_attn_desc(kernel_shape=KERNEL_SHAPE, num_requests=case.B, num_q_heads=case.Hq, num_kv_heads=case.Hkv, head_dim=case.D,
                            gamma=case.gamma, branch_len=case.L, block_size=case.block_size,
                            max_blocks_per_request=case.max_blocks, q_dtype=case.q_dtype, kv_dtype=case.kv_dtype,
                            branch_kv_dtype=case.branch_kv_dtype, out_dtype=case.out_dtype,
                            softmax_scale=case.scale if scale is None else scale, kv_split_tokens=kv_split_tokens)


def run_attention(case: W.AttnCase, inp: dict, kv_split_tokens: int = 0, want_lse: bool = True, dev=None, scale=None):
    """Returns (out, lse) as fp64 numpy arrays [B,gamma,L,Hq,D], [B,gamma,L,Hq]."""
    dev = dev or upload_attention(case, inp)
    desc = attn_desc(case, kv_split_tokens, scale)
    lens = [int(x) for x in inp["prefix_lens"]]
    ws_bytes = B.la_verify_attention_workspace(desc, lens)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    out = B.empty_out((case.B, case.gamma, case.L, case.Hq, case.D), case.out_dtype)
    out.fill_(float("nan"))
    lse = torch.full((case.B, case.gamma, case.L, case.Hq), float("nan"), dtype=torch.float32, device="cuda") \
        if want_lse else None
    B.la_verify_attention(desc, dev["q"], dev["k_cache"], dev["v_cache"], dev["block_tables"], dev["prefix_lens"],
                          lens, dev["k_branch"], dev["v_branch"], dev["k_scale"], dev["v_scale"], out, lse, ws)
    torch.cuda.synchronize()
    return out.double().cpu().numpy(), (None if lse is None else lse.double().cpu().numpy())


def run_attention_nested(case: W.AttnCase, inp: dict, chain: dict, kv_split_tokens: int = 0):
    """la_verify_attention_nested on ``inp`` plus the drafted chain ``chain`` (k_chain, v_chain, chain_vis)."""
    dev = upload_attention(case, inp)
    desc = attn_desc(case, kv_split_tokens)
    lens = [int(x) for x in inp["prefix_lens"]]
    ws = torch.empty(max(B.la_verify_attention_workspace(desc, lens), 16), dtype=torch.uint8, device="cuda")
    out = B.empty_out((case.B, case.gamma, case.L, case.Hq, case.D), case.out_dtype)
    out.fill_(float("nan"))
    lse = torch.full((case.B, case.gamma, case.L, case.Hq), float("nan"), dtype=torch.float32, device="cuda")
    has = chain["k_chain"].shape[1] > 0
    kch = B.to_device(chain["k_chain"], case.branch_kv_dtype) if has else None
    vch = B.to_device(chain["v_chain"], case.branch_kv_dtype) if has else None
    vis = torch.from_numpy(chain["chain_vis"]).cuda() if has else None
    B.la_verify_attention_nested(desc, dev["q"], dev["k_cache"], dev["v_cache"], dev["block_tables"],
                                 dev["prefix_lens"], lens, dev["k_branch"], dev["v_branch"], kch, vch, vis,
                                 chain["chain_vis"].tolist(), dev["k_scale"], dev["v_scale"], out, lse, ws)
    torch.cuda.synchronize()
    return out.double().cpu().numpy(), lse.double().cpu().numpy()


def run_attention_tree(case: W.AttnCase, inp: dict, tree: dict, kv_split_tokens: int = 0):
    """la_verify_attention_tree on ``inp`` plus the pool ``tree`` (k_pool, v_pool, pool_seg, seg_mask)."""
    dev = upload_attention(case, inp)
    desc = attn_desc(case, kv_split_tokens)
    lens = [int(x) for x in inp["prefix_lens"]]
    ws = torch.empty(max(B.la_verify_attention_workspace(desc, lens), 16), dtype=torch.uint8, device="cuda")
    out = B.empty_out((case.B, case.gamma, case.L, case.Hq, case.D), case.out_dtype)
    out.fill_(float("nan"))
    lse = torch.full((case.B, case.gamma, case.L, case.Hq), float("nan"), dtype=torch.float32, device="cuda")
    has = tree["k_pool"].shape[1] > 0
    kp = B.to_device(tree["k_pool"], case.branch_kv_dtype) if has else None
    vp = B.to_device(tree["v_pool"], case.branch_kv_dtype) if has else None
    seg = torch.from_numpy(tree["pool_seg"]).cuda() if has else None
    mask = torch.from_numpy(tree["seg_mask"].view(np.int64)).cuda() if has else None
    B.la_verify_attention_tree(desc, dev["q"], dev["k_cache"], dev["v_cache"], dev["block_tables"],
                               dev["prefix_lens"], lens, dev["k_branch"], dev["v_branch"], kp, vp, seg,
                               tree["pool_seg"].tolist(), mask, dev["k_scale"], dev["v_scale"], out, lse, ws)
    torch.cuda.synchronize()
    return out.double().cpu().numpy(), lse.double().cpu().numpy()


def row_errors(got: np.ndarray, ref: np.ndarray):
    """Per output row: max |got-ref| over D divided by max |ref| over D.  Returns the vector of row errors."""
    D = ref.shape[-1]
    g, r = got.reshape(-1, D), ref.reshape(-1, D)
    return np.abs(g - r).max(axis=1) / np.abs(r).max(axis=1)


def elem_errors(got: np.ndarray, ref: np.ndarray, floor: float = 1e-3):
    """Element-wise relative error |got-ref| / max(|ref|, floor * max|ref| over the row), the companion figure of
    the row error: reported, not bounded (an element a thousand times smaller than its row's largest is compared
    against that floor).  Returns the array of element errors."""
    D = ref.shape[-1]
    g, r = got.reshape(-1, D), ref.reshape(-1, D)
    den = np.maximum(np.abs(r), floor * np.abs(r).max(axis=1, keepdims=True))
    return np.abs(g - r) / den


def error_report(got: np.ndarray, ref: np.ndarray) -> dict:
    """Both error figures of one comparison, for logs and the benchmark's JSON."""
    row = row_errors(got, ref)
    el = elem_errors(got, ref)
    return {"rows": int(row.size), "max_row_err": float(row.max()), "mean_row_err": float(row.mean()),
            "max_elem_rel_err_floor_1e-3": float(el.max()), "p999_elem_rel_err": float(np.quantile(el, 0.999)),
            "median_elem_rel_err": float(np.median(el))}


def upload_accept(case: W.AcceptCase, inp: dict) -> dict:
    return {
        "target_logits": B.to_device(inp["target_logits"], case.logits_dtype),
        "draft_logits": B.to_device(inp["draft_logits"], case.logits_dtype),
        "draft_tokens": torch.from_numpy(inp["draft_tokens"]).cuda(),
        "u_accept": torch.from_numpy(inp["u_accept"]).cuda(),
        "u_sample": torch.from_numpy(inp["u_sample"]).cuda(),
    }


def run_accept(case: W.AcceptCase, inp: dict, dev=None):
    dev = dev or upload_accept(case, inp)
    desc = B.make_accept_desc(num_branches=case.NB, num_draft=case.K, vocab=case.V, logits_dtype=case.logits_dtype,
                              temperature=case.temperature, top_k=case.top_k, top_p=case.top_p)
    ws = torch.empty(max(B.la_spec_accept_workspace(desc), 16), dtype=torch.uint8, device="cuda")
    n = torch.full((case.NB,), -7, dtype=torch.int32, device="cuda")
    tok = torch.full((case.NB,), -7, dtype=torch.int32, device="cuda")
    ratio = torch.full((case.NB, case.K), float("nan"), dtype=torch.float32, device="cuda")
    B.la_spec_accept(desc, dev["target_logits"], dev["draft_logits"], dev["draft_tokens"], dev["u_accept"],
                     dev["u_sample"], n, tok, ratio, ws)
    torch.cuda.synchronize()
    return {"accepted_len": n.cpu().numpy(), "next_token": tok.cpu().numpy(), "ratio": ratio.double().cpu().numpy()}


def compare_accept(got: dict, ref: dict, threshold_eps: float = 1e-6):
    """Bit-exact comparison of (n, token) with the oracle.  A branch is set aside (counted, not compared) when one of
    its examined accept draws lies within threshold_eps of the min(1, p/q) threshold in the oracle's fp64 -- the
    benchmark's stated exception -- or when a top-p cut of one of its target rows lies within 1e-9 (relative mass) of
    a token boundary, where two fp64 summation orders may differ.  The sampled token needs no exception: both sides
    walk the resampling row in fp64.  Returns (branches whose n differs, branches with equal n whose token differs,
    branches set aside)."""
    NB = ref["accepted_len"].shape[0]
    near_thr = np.zeros(NB, dtype=bool)
    for nb in range(NB):
        examined = np.isfinite(ref["margin"][nb])
        near_thr[nb] = bool((ref["margin"][nb][examined] <= threshold_eps).any())
    # a top-p decision closer than 1e-9 (relative mass) to its threshold may fall either way between two fp64
    # summation orders; such branches are set aside too
    near_thr |= ref["warp_margin"] < 1e-9
    clean = ~near_thr
    bad_n = clean & (got["accepted_len"] != ref["accepted_len"])
    same_n = clean & ~bad_n
    bad_tok = same_n & (got["next_token"] != ref["next_token"])
    return int(bad_n.sum()), int(bad_tok.sum()), int(near_thr.sum())
