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
    out = {"attention": {}, "accept": {}}
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
    return out


if __name__ == "__main__":
    path = Path(__file__).with_name("oracle_small_cases.json")
    path.write_text(json.dumps(compute(), indent=1) + "\n")
    print("wrote", path)
