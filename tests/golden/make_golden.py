"""Writes tests/golden/oracle_small_cases.json: outputs of the CPU oracle on small seeded problems.

The values stored there come from ``oracle/`` only (never from the GPU path); the test that reads the file
(tests/test_golden.py) recomputes them and so notices any later change of the oracle's arithmetic.  What makes the
oracle itself trustworthy are the pins in tests/test_oracle_*.py; this file only freezes it.

Run from the repository root:  python tests/golden/make_golden.py
"""
import json
import sys
from pathlib import Path

import numpy as np

ROOT = Path(__file__).resolve().parents[2]
sys.path.insert(0, str(ROOT))

import oracle  # noqa: E402
from oracle import planner  # noqa: E402
from paper_2506_19830_amd import workloads as W  # noqa: E402  (seeded input generators only)

ATTN = [
    W.AttnCase("golden_f32", (37, 5), 2, 3, 4, 2, 64, "f32", "f32", "f32", "f32", paged=True, seed=101),
    W.AttnCase("golden_fp8", (50,), 3, 2, 4, 1, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16", seed=102),
]
ACCEPT = [
    W.AcceptCase("golden_dense", 6, 3, 97, "f32", target_std=2.0, draft_noise_std=0.8, seed=103),
    W.AcceptCase("golden_lookup_warped", 6, 3, 97, "f32", temperature=0.6, top_k=20, top_p=0.95, point_mass=True,
                 peak=4.0, seed=104),
]


def compute():
    out = {"attention": {}, "accept": {}, "nested": {}, "tree": {}, "commit": {}, "planner": {}}
    for c in ATTN:
        inp = W.make_attention_inputs(c)
        o, lse = oracle.verify_attention(**inp, q_dtype=c.q_dtype, kv_dtype=c.kv_dtype,
                                         branch_kv_dtype=c.branch_kv_dtype, block_size=c.block_size, scale=c.scale)
        out["attention"][c.name] = {"out_first_row": o.reshape(-1, c.D)[0].tolist(),
                                    "out_last_row": o.reshape(-1, c.D)[-1].tolist(),
                                    "out_sum": float(o.sum()), "lse": lse.reshape(-1).tolist()}
    for c in ACCEPT:
        inp = W.make_accept_inputs(c)
        r = oracle.spec_accept(**inp, logits_dtype=c.logits_dtype, temperature=c.temperature, top_k=c.top_k,
                               top_p=float(np.float32(c.top_p)))
        out["accept"][c.name] = {"accepted_len": r["accepted_len"].tolist(), "next_token": r["next_token"].tolist(),
                                 "cdf_lo": r["cdf_lo"].tolist(), "cdf_hi": r["cdf_hi"].tolist()}
    # nested and tree forms, KV commit: the first attention case and a bf16 -> fp8 case with spare cache room
    c = ATTN[0]
    inp = W.make_attention_inputs(c)
    kw = dict(q_dtype=c.q_dtype, kv_dtype=c.kv_dtype, branch_kv_dtype=c.branch_kv_dtype, block_size=c.block_size,
              scale=c.scale)
    chain = W.make_chain_inputs(c, 7, inp, np.array([[0, 7], [3, 5]], dtype=np.int32))
    o, lse = oracle.verify_attention(**inp, **chain, **kw)
    out["nested"][c.name] = {"out_sum": float(o.sum()), "out_last_row": o.reshape(-1, c.D)[-1].tolist(),
                             "lse": lse.reshape(-1).tolist()}
    tree = W.make_tree_inputs(c, 2, 2, 3, inp)
    o, lse = oracle.verify_attention(**inp, **tree, **kw)
    out["tree"][c.name] = {"out_sum": float(o.sum()), "out_last_row": o.reshape(-1, c.D)[-1].tolist(),
                           "lse": lse.reshape(-1).tolist(), "seg_mask": [int(m) for m in tree["seg_mask"].reshape(-1)]}
    cc = W.AttnCase("golden_commit", (21, 4), 2, 5, 2, 2, 32, "bf16", "fp8_e4m3", "bf16", "bf16", seed=105,
                    spare_tokens=16)
    inp = W.make_attention_inputs(cc)
    chain = W.make_chain_inputs(cc, 6, inp)
    kc, vc, new_lens = oracle.kv_commit(inp["k_cache"], inp["v_cache"], None, inp["prefix_lens"], inp["k_branch"],
                                        inp["v_branch"], chain["k_chain"], chain["v_chain"], [1, 0], [6, 2], [5, 3],
                                        inp["k_scale"], inp["v_scale"], kv_dtype="fp8_e4m3", branch_kv_dtype="bf16",
                                        block_size=cc.block_size)
    out["commit"][cc.name] = {"new_lens": new_lens.tolist(), "k_bytes_sum": int(kc.astype(np.int64).sum()),
                              "v_bytes_sum": int(vc.astype(np.int64).sum()),
                              "k_token_21_head_0": kc[1, 0, 21 - 16].tolist(),   # first appended token of request 0
                              "v_token_5_head_1_req_1": vc[cc.max_blocks, 1, 5].tolist()}
    tree = W.make_tree_inputs(cc, 2, 2, 2, inp)                                      # 6 nodes of 2 tokens
    kc, vc, new_lens = oracle.kv_commit_tree(inp["k_cache"], inp["v_cache"], None, inp["prefix_lens"], inp["k_branch"],
                                             inp["v_branch"], tree["k_pool"], tree["v_pool"], tree["pool_seg"],
                                             [0b100010, 0b000001], [1, 0], [5, 3], inp["k_scale"], inp["v_scale"],
                                             kv_dtype="fp8_e4m3", branch_kv_dtype="bf16", block_size=cc.block_size)
    out["commit"][cc.name + "_tree"] = {"new_lens": new_lens.tolist(), "k_bytes_sum": int(kc.astype(np.int64).sum()),
                                        "v_bytes_sum": int(vc.astype(np.int64).sum()),
                                        "k_token_23_head_0": kc[1, 0, 23 - 16].tolist()}   # first token of node 5
    walks = planner.tree_output_construction([-1, -1, 0, 0, 1, 1], [[0, 1, 1, 1, 0, 1], [1, 1, 0, 0, 1, 1]],
                                             [[3, 4, 5, 6, 7, 8, 9]] * 2)
    out["planner"]["tree_walk"] = {k: [w[i] for w in walks]
                                   for i, k in enumerate(("depth", "src_branch", "commit_mask", "n_own"))}
    # controller / planner (Section 3.2, 3.3): the parameters of the theorem's range and one outside it
    for name, (a1, c1, a2, c2, m, asyn) in {"hybrid_async": (0.7, 0.2, 0.65, 0.1, 16, True),
                                            "hybrid_sync": (0.7, 0.2, 0.65, 0.1, 16, False),
                                            "low_acceptance": (0.2, 0.45, 0.3, 0.3, 8, True)}.items():
        k1, k2, h, _ = planner.plan(a1, c1, a2, c2, m, asyn)
        out["planner"][name] = {"k1": k1, "k2": k2, "h": h, "f_sync_4": planner.speedup_sync(a1, c1, 4),
                                "f_async_3": planner.speedup_async(a1, c1, 3), "f_async_9": planner.speedup_async(a1, c1, 9)}
    return out


if __name__ == "__main__":
    path = Path(__file__).with_name("oracle_small_cases.json")
    path.write_text(json.dumps(compute(), indent=1) + "\n")
    print("wrote", path)
