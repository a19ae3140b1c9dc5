"""The library under HIP graph capture: its calls allocate nothing, never synchronise and enqueue only kernels on
the caller's stream, so a whole verification step can be captured once and replayed.  Every replay is checked
against an eager run on the same (changed in place between replays) inputs."""
import numpy as np
import pytest
import torch

from paper_2506_19830_amd import binding as B
from paper_2506_19830_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_captured_step_replays_like_eager():
    from gpu_util import attn_desc, upload_accept, upload_attention
    case = W.AttnCase("graph", (700, 64), 3, 9, 8, 2, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16", paged=True,
                      seed=81, spare_tokens=64)
    acase = W.AcceptCase("graph_accept", 6, 4, 8193, "bf16", seed=82)
    inp = W.make_attention_inputs(case)
    chain = W.make_chain_inputs(case, 20, inp)
    dev = upload_attention(case, inp)
    kch, vch = B.to_device(chain["k_chain"], "fp8_e4m3"), B.to_device(chain["v_chain"], "fp8_e4m3")
    vis = torch.from_numpy(chain["chain_vis"]).cuda()
    acc = upload_accept(acase, W.make_accept_inputs(acase))
    lens = [int(x) for x in case.prefix_lens]
    desc = attn_desc(case)
    adesc = B.make_accept_desc(num_branches=acase.NB, num_draft=acase.K, vocab=acase.V, logits_dtype="bf16")
    ws = torch.empty(max(16, B.la_verify_attention_workspace(desc, lens)), dtype=torch.uint8, device="cuda")
    aws = torch.empty(max(16, B.la_spec_accept_workspace(adesc)), dtype=torch.uint8, device="cuda")
    shape = (case.B, case.gamma, case.L, case.Hq, case.D)
    src = torch.tensor([1, 2], dtype=torch.int32, device="cuda")
    nch = torch.tensor([6, 13], dtype=torch.int32, device="cuda")
    nown = torch.tensor([9, 4], dtype=torch.int32, device="cuda")

    def step(out, out_nested, n_acc, tok, new_lens, k_cache, v_cache):
        B.la_verify_attention(desc, dev["q"], k_cache, v_cache, dev["block_tables"], dev["prefix_lens"], lens,
                              dev["k_branch"], dev["v_branch"], dev["k_scale"], dev["v_scale"], out, None, ws)
        B.la_verify_attention_nested(desc, dev["q"], k_cache, v_cache, dev["block_tables"], dev["prefix_lens"], lens,
                                     dev["k_branch"], dev["v_branch"], kch, vch, vis, chain["chain_vis"].tolist(),
                                     dev["k_scale"], dev["v_scale"], out_nested, None, ws)
        B.la_spec_accept(adesc, acc["target_logits"], acc["draft_logits"], acc["draft_tokens"], acc["u_accept"],
                         acc["u_sample"], n_acc, tok, None, aws)
        B.la_kv_commit(desc, k_cache, v_cache, dev["block_tables"], dev["prefix_lens"], lens, dev["k_branch"],
                       dev["v_branch"], kch, vch, src, nch, nown, dev["k_scale"], dev["v_scale"], new_lens)

    def buffers():
        return (B.empty_out(shape, "bf16"), B.empty_out(shape, "bf16"),
                torch.zeros(acase.NB, dtype=torch.int32, device="cuda"),
                torch.zeros(acase.NB, dtype=torch.int32, device="cuda"),
                torch.zeros(case.B, dtype=torch.int32, device="cuda"), dev["k_cache"].clone(), dev["v_cache"].clone())

    graph_bufs, eager_bufs = buffers(), buffers()
    step(*graph_bufs)                                   # warm-up outside the capture (module loading, attributes)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(*graph_bufs)
    rng = np.random.default_rng(0)
    for replay in range(4):
        # change the inputs in place between replays (eager work and a synchronisation in between)
        dev["q"].copy_(torch.from_numpy(rng.standard_normal(shape).astype(np.float32)).cuda().to(torch.bfloat16))
        acc["u_accept"].copy_(torch.from_numpy(rng.random((acase.NB, acase.K), dtype=np.float32)).cuda())
        for t in graph_bufs[:5] + eager_bufs[:5]:
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        step(*eager_bufs)
        torch.cuda.synchronize()
        for g, e in zip(graph_bufs, eager_bufs):
            assert torch.equal(g.view(torch.uint8) if g.dtype == torch.float8_e4m3fn else g,
                               e.view(torch.uint8) if e.dtype == torch.float8_e4m3fn else e), f"replay {replay}"
        assert graph_bufs[4].tolist() == [700 + 6 + 9, 64 + 13 + 4]


@pytest.mark.parametrize("top_k", [20, 0])
def test_captured_accept_with_warped_targets_replays_like_eager(top_k):
    """la_spec_accept with temperature, top-k / top-p and prompt-lookup drafts (the slice-sum kernel, the candidate
    lists in LDS, the list sort) captured once and replayed on uniforms and logits changed in place: every replay
    equals an eager run, and they are not all the same."""
    from gpu_util import upload_accept
    acase = W.AcceptCase("graph_warp", 6, 3, 40000, "bf16", temperature=0.6, top_k=top_k, top_p=0.95, point_mass=True,
                         peak=6.0, seed=83)
    acc = upload_accept(acase, W.make_accept_inputs(acase))
    adesc = B.make_accept_desc(num_branches=acase.NB, num_draft=acase.K, vocab=acase.V, logits_dtype="bf16",
                               temperature=acase.temperature, top_k=acase.top_k, top_p=acase.top_p)
    aws = torch.empty(max(16, B.la_spec_accept_workspace(adesc)), dtype=torch.uint8, device="cuda")

    def step(n_acc, tok, ratio):
        B.la_spec_accept(adesc, acc["target_logits"], acc["draft_logits"], acc["draft_tokens"], acc["u_accept"],
                         acc["u_sample"], n_acc, tok, ratio, aws)

    def buffers():
        return (torch.zeros(acase.NB, dtype=torch.int32, device="cuda"),
                torch.zeros(acase.NB, dtype=torch.int32, device="cuda"),
                torch.zeros((acase.NB, acase.K), dtype=torch.float32, device="cuda"))

    graph_bufs, eager_bufs = buffers(), buffers()
    step(*graph_bufs)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(*graph_bufs)
    rng = np.random.default_rng(1)
    seen = set()
    for replay in range(4):
        acc["u_accept"].copy_(torch.from_numpy(rng.random((acase.NB, acase.K), dtype=np.float32)).cuda())
        acc["u_sample"].copy_(torch.from_numpy(rng.random(acase.NB, dtype=np.float32)).cuda())
        acc["target_logits"].copy_(acc["target_logits"].roll(replay + 1, dims=0))     # the branches' rows change places
        for t in graph_bufs + eager_bufs:
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        step(*eager_bufs)
        torch.cuda.synchronize()
        for g, e in zip(graph_bufs, eager_bufs):
            assert torch.equal(g, e), f"replay {replay}"
        seen.add((tuple(graph_bufs[0].tolist()), tuple(graph_bufs[1].tolist())))
    assert len(seen) > 1
