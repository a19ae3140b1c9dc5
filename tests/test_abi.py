"""The C-ABI library without a GPU: it loads, exports every symbol the header declares, and rejects bad
arguments on the host before anything is launched (these calls never reach a kernel)."""
import ctypes
import re
from pathlib import Path

import pytest

from paper_2506_19830_amd import binding as B

ROOT = Path(__file__).resolve().parent.parent


def good_desc(**kw):
    d = dict(num_requests=1, num_q_heads=40, num_kv_heads=8, head_dim=128, gamma=8, branch_len=64, block_size=16,
             max_blocks_per_request=2048, q_dtype="bf16", kv_dtype="fp8_e4m3", branch_kv_dtype="fp8_e4m3",
             out_dtype="bf16", softmax_scale=128 ** -0.5)
    d.update(kw)
    return B.make_attn_desc(**d)


def _declared(header_name):
    header = (ROOT / "include" / header_name).read_text()
    return set(re.findall(r"LA_API[^;(]*?\b(la_\w+)\s*\(", header))


def _exported(path):
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", str(path)], capture_output=True, text=True, check=True).stdout
    return {line.split()[-1] for line in out.splitlines() if " T " in line}


def test_library_exports_every_declared_symbol():
    """The product library exports exactly what la_verify.h declares; the benchmark library that and the aids of
    la_verify_bench.h; neither exports anything else."""
    declared = _declared("la_verify.h")
    aids = _declared("la_verify_bench.h")
    assert declared == set(B.EXPORTED_SYMBOLS) and aids == set(B.BENCH_SYMBOLS)
    lib, bench = B.load("product"), B.load("bench")
    for name in declared:
        assert hasattr(lib, name) and hasattr(bench, name), name
    for name in aids:
        assert hasattr(bench, name) and not hasattr(lib, name), name
    assert _exported(B.LIB_PATH) == declared
    assert _exported(B.BENCH_LIB_PATH) == declared | aids


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(B.la_attn_desc) == 15 * 4
    assert ctypes.sizeof(B.la_attn_plan) == 7 * 4
    assert ctypes.sizeof(B.la_accept_desc) == 7 * 4
    assert ctypes.sizeof(B.la_layer_strides) == 8 + 4 * 8        # int32 padded to the int64 that follows


def test_status_strings():
    assert B.status_string(0) == "ok"
    assert "workspace" in B.status_string(3)
    assert B.status_string(99) == "unknown status"


def test_workspace_query_and_plan():
    ws = B.la_verify_attention_workspace(good_desc(), [32768])
    rows = 8 * 64 * 40
    assert ws > 0 and ws % (rows * 130 * 4) < 512          # whole partial slots (O[128] + m + l per row)
    assert B.la_verify_attention_workspace(good_desc(kv_split_tokens=32768), [32768]) < ws
    f32 = good_desc(q_dtype="f32", kv_dtype="f32", branch_kv_dtype="f32", out_dtype="f32", head_dim=64)
    assert B.la_verify_attention_workspace(f32, [32768]) == 0
    acc = B.make_accept_desc(num_branches=8, num_draft=8, vocab=152064, logits_dtype="bf16")
    assert B.la_spec_accept_workspace(acc) > 8 * 17 * 19 * 8


def test_planner_deals_unequal_requests_as_the_hardware_does():
    """Configuration 4's batch: four requests of 8K..32K keys on a bf16 cache, 3072 rows per KV head.  One chunk per
    request and chunks of a quarter of the longest need the same number of rounds x longest-chunk steps; dealt out in
    launch order the first leaves the chip half empty while the longest request runs (measured 1.17 against 1.04 ms).
    The plan must be the balanced one; a single request keeps the plan that rounds x longest gives."""
    kw = dict(num_requests=4, num_q_heads=64, num_kv_heads=8, gamma=8, branch_len=48, kv_dtype="bf16",
              branch_kv_dtype="bf16", max_blocks_per_request=2060)
    plan = B.la_verify_attention_plan(good_desc(**kw), [8192, 16384, 24576, 32768])
    assert plan["chunk_tokens"] == 8192 and plan["chunks_total"] == 10
    one = B.la_verify_attention_plan(good_desc(), [32768])
    assert one["kernel_shape"] == 1 and one["chunk_tokens"] == 10944 and one["workgroups"] == 240
    # every la_verify_attention call plans on the host before it enqueues anything: the plan must stay cheap
    import time
    few_rows = good_desc(num_requests=4, branch_len=4, max_blocks_per_request=2060)
    t0 = time.perf_counter()
    for _ in range(50):
        B.la_verify_attention_plan(few_rows, [8192, 16384, 24576, 32768])
    assert (time.perf_counter() - t0) / 50 < 5e-4          # observed 13 us; an allocating version of the model took 3 ms


@pytest.mark.parametrize("kw,lens,status", [
    (dict(num_q_heads=41), [100], 1),
    (dict(block_size=8), [100], 1),
    (dict(softmax_scale=0.0), [100], 1),
    (dict(kv_split_tokens=100), [100], 1),
    (dict(gamma=0), [100], 1),
    (dict(), [-1], 1),
    (dict(max_blocks_per_request=4), [65], 1),
    (dict(head_dim=96), [100], 2),
    (dict(head_dim=64, kernel_shape=1), [100], 2),
    (dict(q_dtype="f32"), [100], 2),
    (dict(kv_dtype="bf16", branch_kv_dtype="fp8_e4m3"), [100], 2),
    (dict(out_dtype="fp8_e4m3"), [100], 2),
])
def test_attention_rejects_bad_descriptors(kw, lens, status):
    with pytest.raises(B.LaError) as e:
        B.la_verify_attention_workspace(good_desc(**kw), lens)
    assert e.value.status == status


def _call_attention(desc, lens, ptrs, ws_bytes):
    lib = B.load()
    arr = (ctypes.c_int32 * len(lens))(*lens)
    vp = ctypes.c_void_p
    return lib.la_verify_attention(ctypes.byref(desc), vp(ptrs.get("q", 256)), vp(ptrs.get("k", 256)),
                                   vp(ptrs.get("v", 256)), vp(0), vp(ptrs.get("lens", 256)), arr,
                                   vp(ptrs.get("kb", 256)), vp(ptrs.get("vb", 256)), vp(0), vp(0),
                                   vp(ptrs.get("out", 256)), vp(0), vp(ptrs.get("ws", 256)),
                                   ctypes.c_size_t(ws_bytes), vp(0))


def test_attention_call_rejects_before_launch():
    """Fake (never dereferenced) device addresses: each call must fail validation on the host."""
    d = good_desc()
    assert _call_attention(d, [32768], {"q": 0}, 1 << 40) == 1           # required pointer missing
    assert _call_attention(d, [32768], {"k": 0}, 1 << 40) == 1           # prefix present but no cache
    assert _call_attention(d, [32768], {"out": 264}, 1 << 40) == 1       # not 16-byte aligned
    assert _call_attention(d, [32768], {}, 1024) == 3                    # workspace too small
    assert _call_attention(d, [32768], {"ws": 0}, 0) == 3


def test_nested_attention_call_rejects_before_launch():
    """Chain arguments are validated on the host: length, pointers, alignment, visibility within 0..C."""
    lib = B.load()
    d = good_desc()
    vp = ctypes.c_void_p
    lens = (ctypes.c_int32 * 1)(32768)
    n_vis = d.num_requests * d.gamma

    def call(chain_len, k_chain=256, v_chain=256, vis_dev=256, vis=None, vis_host_null=False, ws_bytes=1024):
        vis_arr = (ctypes.c_int32 * n_vis)(*(vis if vis is not None else [0] * n_vis))
        host = ctypes.POINTER(ctypes.c_int32)() if vis_host_null else vis_arr
        return lib.la_verify_attention_nested(ctypes.byref(d), vp(256), vp(256), vp(256), vp(0), vp(256), lens,
                                              vp(256), vp(256), vp(k_chain), vp(v_chain), ctypes.c_int32(chain_len),
                                              vp(vis_dev), host, vp(0), vp(0), vp(256), vp(0), vp(256),
                                              ctypes.c_size_t(ws_bytes), vp(0))

    assert call(-1) == 1
    assert call(4, k_chain=0) == 1
    assert call(4, v_chain=264) == 1                       # not 16-byte aligned
    assert call(4, vis_dev=0) == 1
    assert call(4, vis_host_null=True) == 1
    assert call(4, vis=[0] * (n_vis - 1) + [5]) == 1       # sees more than the chain holds
    assert call(4, vis=[-1] + [0] * (n_vis - 1)) == 1
    # valid chain arguments get as far as the workspace check (nothing is launched: the workspace is too small)
    assert call(4, vis=[4] * n_vis) == 3
    assert call(0, k_chain=0, v_chain=0, vis_dev=0, vis_host_null=True) == 3


def test_kv_commit_rejects_before_launch():
    lib = B.load()
    vp = ctypes.c_void_p
    lens = (ctypes.c_int32 * 1)(32768)

    def call(desc, chain_len=8, strides=None, **ptrs):
        g = lambda k, dflt=256: vp(ptrs.get(k, dflt))
        return lib.la_kv_commit(ctypes.byref(desc), g("kc"), g("vc"), vp(0), g("lens"), lens, g("kb"), g("vb"),
                                g("kch"), g("vch"), ctypes.c_int32(chain_len), g("src"), g("nch"), g("nown"), vp(0),
                                vp(0), g("new", 512), ctypes.byref(strides) if strides is not None else None, vp(0))

    roomy = good_desc(max_blocks_per_request=2048 + 8)           # 32768 + 128 positions
    assert call(good_desc()) == 1                                # table maps exactly the prefix: no room
    assert call(roomy, kc=0) == 1
    assert call(roomy, kch=0) == 1                               # chain_len 8 without a chain
    assert call(roomy, chain_len=-1) == 1
    assert call(roomy, kb=264) == 1                              # not 16-byte aligned
    assert call(roomy, new=256, lens=256) == 1                   # new lengths alias the old ones
    assert call(good_desc(max_blocks_per_request=2048 + 8, kv_dtype="bf16", branch_kv_dtype="bf16",
                          head_dim=100)) == 2
    assert call(good_desc(max_blocks_per_request=2048 + 8, q_dtype="f32", kv_dtype="f32",
                          branch_kv_dtype="bf16", out_dtype="f32")) == 2   # no such conversion
    bad = B.la_layer_strides(num_layers=0)
    assert call(roomy, strides=bad) == 1
    odd = B.la_layer_strides(num_layers=2, cache_stride=1 << 20, branch_stride=7, chain_stride=1 << 10)
    assert call(roomy, strides=odd) == 1                         # layer 1 of the branch tensors would be unaligned


def test_kv_commit_tree_rejects_before_launch():
    lib = B.load()
    vp = ctypes.c_void_p
    lens = (ctypes.c_int32 * 1)(32768)

    def call(desc, pool_len=8, **ptrs):
        g = lambda k, dflt=256: vp(ptrs.get(k, dflt))
        return lib.la_kv_commit_tree(ctypes.byref(desc), g("kc"), g("vc"), vp(0), g("lens"), lens, g("kb"), g("vb"),
                                     g("kp"), g("vp"), ctypes.c_int32(pool_len), g("seg"), g("mask"), g("src"),
                                     g("nown"), vp(0), vp(0), g("new", 512), None, vp(0))

    roomy = good_desc(max_blocks_per_request=2048 + 8)
    assert call(good_desc()) == 1                                # no room behind the prefix
    assert call(roomy, mask=0) == 1
    assert call(roomy, mask=260) == 1                            # 64-bit masks on a 4-byte boundary
    assert call(roomy, seg=0) == 1                               # a pool without node labels
    assert call(roomy, kp=0) == 1
    assert call(roomy, pool_len=-1) == 1
    assert call(roomy, src=0) == 1
    assert call(roomy, new=256, lens=256) == 1


def test_accept_rejects_bad_arguments():
    for kw, status in [(dict(num_branches=0), 1), (dict(num_draft=0), 1), (dict(vocab=0), 1),
                       (dict(temperature=0.0), 1), (dict(logits_dtype="fp8_e4m3"), 2),
                       (dict(num_branches=40000, num_draft=8), 2), (dict(top_k=-1), 1), (dict(top_p=0.0), 1),
                       (dict(top_p=1.5), 1)]:
        base = dict(num_branches=8, num_draft=8, vocab=152064, logits_dtype="bf16")
        base.update(kw)
        with pytest.raises(B.LaError) as e:
            B.la_spec_accept_workspace(B.make_accept_desc(**base))
        assert e.value.status == status
    lib = B.load()
    d = B.make_accept_desc(num_branches=8, num_draft=8, vocab=152064, logits_dtype="bf16")
    vp = ctypes.c_void_p
    args = [vp(256)] * 7 + [vp(0)]
    assert lib.la_spec_accept(ctypes.byref(d), *args, vp(256), ctypes.c_size_t(16), vp(0)) == 3
    args[0] = vp(0)
    assert lib.la_spec_accept(ctypes.byref(d), *args, vp(256), ctypes.c_size_t(1 << 30), vp(0)) == 1


def test_product_package_does_not_import_the_oracle():
    for f in (ROOT / "paper_2506_19830_amd").rglob("*"):
        if f.suffix in (".py", ".hip", ".hpp", ".h", ".cpp"):
            text = f.read_text()
            assert "import oracle" not in text and "from oracle" not in text and "la_oracle" not in text, f
