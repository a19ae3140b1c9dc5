"""The index checkers of the benchmark library (debug aid): the compute calls trust cache block ids and drafted token
ids; these scans find the entries a call would touch that are out of range.  Nothing here hands an out-of-range index
to a compute call: the checkers only read the tables."""
import pytest
import torch

from paper_2506_19830_amd import binding as B
from paper_2506_19830_amd import workloads as W

pytestmark = pytest.mark.gpu


def _desc(case):
    return B.make_attn_desc(num_requests=case.B, num_q_heads=case.Hq, num_kv_heads=case.Hkv, head_dim=case.D,
                            gamma=case.gamma, branch_len=case.L, block_size=case.block_size,
                            max_blocks_per_request=case.max_blocks, q_dtype=case.q_dtype, kv_dtype=case.kv_dtype,
                            branch_kv_dtype=case.branch_kv_dtype, out_dtype=case.out_dtype, softmax_scale=case.scale)


def test_block_table_check_finds_planted_entries_and_only_those():
    case = W.AttnCase("paged", (777, 0, 5, 2049), 2, 17, 8, 2, 128, paged=True, seed=3)
    t = W.make_attention_inputs_device(case, "cuda:0")
    lens = [int(x) for x in case.prefix_lens]
    n_blocks = t["k_cache"].shape[0]
    report = torch.full((3,), 7, dtype=torch.int32, device="cuda")
    desc = _desc(case)
    B.la_check_block_tables(desc, t["block_tables"], lens, n_blocks, report)
    assert report.tolist() == [0, -1, -1]                       # the generator's table is clean
    table = t["block_tables"].clone()
    table[3, 100] = n_blocks                                     # one past the pool, inside request 3's 129 blocks
    table[0, 48] = -1                                            # request 0 uses blocks 0..48
    table[0, 49] = 10 ** 6                                       # past its prefix: never touched, not an offender
    table[1, 0] = -5                                             # request 1 has no prefix: never touched
    B.la_check_block_tables(desc, table, lens, n_blocks, report)
    count, b, j = report.tolist()
    assert count == 2 and (b, j) in ((3, 100), (0, 48))
    B.la_check_block_tables(desc, table, lens, n_blocks, report, extra_tokens=8)    # one more block for requests 0 and 1
    assert report.tolist()[0] == 4
    # a contiguous cache: the identity ids against the pool size
    B.la_check_block_tables(desc, None, lens, case.B * case.max_blocks, report)
    assert report.tolist() == [0, -1, -1]
    B.la_check_block_tables(desc, None, lens, 3 * case.max_blocks + 100, report)     # request 3 needs 129 blocks
    assert report.tolist()[0] == 29 and report.tolist()[1] == 3
    with pytest.raises(B.LaError):
        B.la_check_block_tables(desc, table, [lens[0], lens[1], lens[2], case.max_blocks * 16 + 1], n_blocks, report)


def test_draft_token_check():
    acc = W.AcceptCase("chk", 5, 70, 1000, "f32", seed=2)
    desc = B.make_accept_desc(num_branches=acc.NB, num_draft=acc.K, vocab=acc.V, logits_dtype=acc.logits_dtype)
    tokens = torch.randint(0, acc.V, (acc.NB, acc.K), dtype=torch.int32, device="cuda")
    report = torch.zeros(3, dtype=torch.int32, device="cuda")
    B.la_check_draft_tokens(desc, tokens, report)
    assert report.tolist() == [0, -1, -1]
    tokens[4, 69] = acc.V
    tokens[2, 0] = -1
    B.la_check_draft_tokens(desc, tokens, report)
    count, b, i = report.tolist()
    assert count == 2 and (b, i) in ((4, 69), (2, 0))
