"""Two callers on two HIP streams at once: the compute entry points keep no state of their own (the workspace is
the caller's), so calls in flight together on different streams, each with its own workspace and outputs, must give
the bits they give one after the other.  Both streams have the default priority."""
import pytest
import torch

from paper_2506_19830_amd import binding as B
from paper_2506_19830_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_calls_on_two_streams_give_the_serial_bits():
    from gpu_util import attn_desc, upload_accept, upload_attention
    ca = W.AttnCase("stream_a", (3000, 700), 4, 24, 16, 4, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16", paged=True,
                    seed=91)
    cb = W.AttnCase("stream_b", (2100,), 6, 16, 8, 2, 128, seed=92, spare_tokens=128)
    acase = W.AcceptCase("stream_accept", 16, 4, 50257, "bf16", seed=93)
    ia, ib = W.make_attention_inputs(ca), W.make_attention_inputs(cb)
    chain = W.make_chain_inputs(cb, 80, ib)
    da, db = upload_attention(ca, ia), upload_attention(cb, ib)
    kch, vch = B.to_device(chain["k_chain"], "bf16"), B.to_device(chain["v_chain"], "bf16")
    vis = torch.from_numpy(chain["chain_vis"]).cuda()
    acc = upload_accept(acase, W.make_accept_inputs(acase))
    la, lb = [int(x) for x in ca.prefix_lens], [int(x) for x in cb.prefix_lens]
    desc_a, desc_b = attn_desc(ca), attn_desc(cb)
    adesc = B.make_accept_desc(num_branches=acase.NB, num_draft=acase.K, vocab=acase.V, logits_dtype="bf16")
    src = torch.tensor([3], dtype=torch.int32, device="cuda")
    nch = torch.tensor([48], dtype=torch.int32, device="cuda")
    nown = torch.tensor([16], dtype=torch.int32, device="cuda")

    def buffers():
        return dict(
            ws_a=torch.empty(max(16, B.la_verify_attention_workspace(desc_a, la)), dtype=torch.uint8, device="cuda"),
            ws_b=torch.empty(max(16, B.la_verify_attention_workspace(desc_b, lb)), dtype=torch.uint8, device="cuda"),
            aws=torch.empty(max(16, B.la_spec_accept_workspace(adesc)), dtype=torch.uint8, device="cuda"),
            out_a=B.empty_out((ca.B, ca.gamma, ca.L, ca.Hq, ca.D), "bf16"),
            out_b=B.empty_out((cb.B, cb.gamma, cb.L, cb.Hq, cb.D), "bf16"),
            n_acc=torch.zeros(acase.NB, dtype=torch.int32, device="cuda"),
            tok=torch.zeros(acase.NB, dtype=torch.int32, device="cuda"),
            new_lens=torch.zeros(cb.B, dtype=torch.int32, device="cuda"),
            kc=db["k_cache"].clone(), vc=db["v_cache"].clone())

    def work_a(t):
        B.la_verify_attention(desc_a, da["q"], da["k_cache"], da["v_cache"], da["block_tables"], da["prefix_lens"],
                              la, da["k_branch"], da["v_branch"], da["k_scale"], da["v_scale"], t["out_a"], None,
                              t["ws_a"])
        B.la_spec_accept(adesc, acc["target_logits"], acc["draft_logits"], acc["draft_tokens"], acc["u_accept"],
                         acc["u_sample"], t["n_acc"], t["tok"], None, t["aws"])

    def work_b(t):
        B.la_verify_attention_nested(desc_b, db["q"], t["kc"], t["vc"], None, db["prefix_lens"], lb, db["k_branch"],
                                     db["v_branch"], kch, vch, vis, chain["chain_vis"].tolist(), None, None,
                                     t["out_b"], None, t["ws_b"])
        B.la_kv_commit(desc_b, t["kc"], t["vc"], None, db["prefix_lens"], lb, db["k_branch"], db["v_branch"], kch,
                       vch, src, nch, nown, None, None, t["new_lens"])

    serial = buffers()
    work_a(serial)
    work_b(serial)
    torch.cuda.synchronize()

    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(3):
        both = buffers()
        torch.cuda.synchronize()
        for _ in range(2):                       # the same work twice per stream: the second pass finds the first's
            with torch.cuda.stream(sa):          # outputs and must reproduce them (the commit rewrites the same rows)
                work_a(both)
            with torch.cuda.stream(sb):
                work_b(both)
        torch.cuda.synchronize()
        for key in ("out_a", "out_b", "n_acc", "tok", "new_lens", "kc", "vc"):
            assert torch.equal(both[key].view(torch.uint8), serial[key].view(torch.uint8)), (rep, key)
