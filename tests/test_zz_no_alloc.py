"""The allocation-free form of the accept call (``la_spec_accept_static``) against ``la_spec_accept``: same inputs,
same integers and ratios, on two calls in a row through the C ABI, the second with a smaller input, so that what
the first call left in the library's scratch array must not matter."""
import numpy as np
import pytest
import torch

import gpu_util as U
from paper_2506_19830_amd import binding as B
from paper_2506_19830_amd import workloads as W

pytestmark = pytest.mark.gpu


def _run_static(case, dev):
    desc = B.make_accept_desc(num_branches=case.NB, num_draft=case.K, vocab=case.V, logits_dtype=case.logits_dtype,
                              temperature=case.temperature, top_k=case.top_k, top_p=case.top_p)
    n = torch.full((case.NB,), -7, dtype=torch.int32, device="cuda")
    tok = torch.full((case.NB,), -7, dtype=torch.int32, device="cuda")
    ratio = torch.full((case.NB, case.K), float("nan"), dtype=torch.float32, device="cuda")
    B.la_spec_accept_static(desc, dev["target_logits"], dev["draft_logits"], dev["draft_tokens"], dev["u_accept"],
                            dev["u_sample"], n, tok, ratio)
    torch.cuda.synchronize()
    return {"accepted_len": n.cpu().numpy(), "next_token": tok.cpu().numpy(), "ratio": ratio.double().cpu().numpy()}


def test_static_scratch_matches_workspace_call_twice_in_a_row():
    cases = [
        W.AcceptCase("static_large", 12, 6, 40000, "bf16", seed=31),
        W.AcceptCase("static_small", 3, 2, 5000, "bf16", seed=32),                       # smaller, same dtype
        W.AcceptCase("static_warped", 5, 3, 9000, "f32", temperature=0.6, top_k=20, top_p=0.95, point_mass=True,
                     peak=9.0, seed=33),                                                # other kernels, other dtype
    ]
    for case in cases:
        inp = W.make_accept_inputs(case)
        dev = U.upload_accept(case, inp)
        want = U.run_accept(case, inp, dev)
        got = _run_static(case, dev)
        assert np.array_equal(got["accepted_len"], want["accepted_len"]), case.name
        assert np.array_equal(got["next_token"], want["next_token"]), case.name
        assert np.array_equal(got["ratio"], want["ratio"], equal_nan=True), case.name
        assert (want["accepted_len"] >= 0).all() and (want["next_token"] >= 0).all()


def test_static_scratch_rejects_oversized_problems():
    desc = B.make_accept_desc(num_branches=256, num_draft=8, vocab=152064, logits_dtype="bf16", temperature=1.0,
                              top_k=0, top_p=1.0)
    assert B.la_spec_accept_workspace(desc) > (16 << 20)
    t = torch.zeros(16, dtype=torch.int32, device="cuda")
    with pytest.raises(B.LaError) as err:
        B.la_spec_accept_static(desc, t, t, t, t, t, t, t, None)
    assert err.value.status == 3  # LA_ERR_WORKSPACE_TOO_SMALL
