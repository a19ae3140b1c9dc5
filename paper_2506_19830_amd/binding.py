"""ctypes binding of ``libla_verify.so`` (argument marshalling only).

The functions mirror the C ABI in ``include/la_verify.h`` name for name.  torch
is used for device memory and the current HIP stream, nothing else: every step
of the verification path runs inside the library's kernels.  There is no
fallback -- if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path
from typing import Optional, Sequence

import torch

_HERE = Path(__file__).resolve().parent

# The product library, and the same objects linked together with the benchmark aids (la_verify_bench.h).
LIB_PATH = _HERE / "libla_verify.so"
BENCH_LIB_PATH = _HERE / "libla_verify_bench.so"

LA_F32, LA_BF16, LA_FP8_E4M3 = 0, 1, 2
DTYPE_CODES = {"f32": LA_F32, "bf16": LA_BF16, "fp8_e4m3": LA_FP8_E4M3}
_TORCH_DTYPES = {"f32": torch.float32, "bf16": torch.bfloat16, "fp8_e4m3": torch.float8_e4m3fn}

EXPORTED_SYMBOLS = (
    "la_verify_attention_workspace", "la_verify_attention_plan", "la_verify_attention", "la_verify_attention_nested",
    "la_verify_attention_tree", "la_kv_commit", "la_kv_commit_tree", "la_step_select_tree", "la_step_select",
    "la_speedup_step_sync", "la_speedup_step_async", "la_speedup_token", "la_plan_budget",
    "la_spec_accept_workspace", "la_spec_accept", "la_spec_accept_static", "la_status_string",
)
# what libla_verify_bench.so exports on top of those (la_verify_bench.h)
BENCH_SYMBOLS = (
    "la_calibrate_mfma", "la_calibrate_mfma_data", "la_calibrate_read", "la_calibrate_issue", "la_selftest_exp64", "la_selftest_second_attempt", "la_check_block_tables", "la_check_draft_tokens",
    "la_profile_enable", "la_profile_select",
    "la_profile_collect", "la_profile_num_kernels", "la_profile_get", "la_profile_reset",
)


class la_attn_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "num_requests", "num_q_heads", "num_kv_heads", "head_dim", "gamma", "branch_len", "block_size",
        "max_blocks_per_request", "q_dtype", "kv_dtype", "branch_kv_dtype", "out_dtype")] + [
        ("softmax_scale", ctypes.c_float), ("kv_split_tokens", ctypes.c_int32), ("kernel_shape", ctypes.c_int32)]


class la_attn_plan(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "path", "kernel_shape", "rows_per_workgroup", "row_tiles", "chunk_tokens", "chunks_total", "workgroups")]


class la_accept_desc(ctypes.Structure):
    _fields_ = [("num_branches", ctypes.c_int32), ("num_draft", ctypes.c_int32), ("vocab", ctypes.c_int32),
                ("logits_dtype", ctypes.c_int32), ("temperature", ctypes.c_float), ("top_k", ctypes.c_int32),
                ("top_p", ctypes.c_float)]


class la_layer_strides(ctypes.Structure):
    _fields_ = [("num_layers", ctypes.c_int32), ("cache_stride", ctypes.c_int64), ("branch_stride", ctypes.c_int64),
                ("chain_stride", ctypes.c_int64), ("scale_stride", ctypes.c_int64)]


class la_plan_desc(ctypes.Structure):
    _fields_ = [("alpha1", ctypes.c_double), ("c1", ctypes.c_double), ("alpha2", ctypes.c_double),
                ("c2", ctypes.c_double), ("budget", ctypes.c_int32), ("asynchronous", ctypes.c_int32)]


class LaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_libs = {}
_active = "product"


def select_library(kind: str) -> None:
    """Route every call of this module through the product library (``"product"``, the default) or through the
    benchmark build (``"bench"``: the same objects plus the aids of ``la_verify_bench.h``; needed for
    ``la_profile_*`` to see the launches)."""
    global _active
    if kind not in ("product", "bench"):
        raise ValueError(kind)
    _active = kind


def load(kind: Optional[str] = None) -> ctypes.CDLL:
    """Load the HIP library; raises if it was not built (there is no other implementation)."""
    kind = kind or _active
    if kind not in _libs:
        path = LIB_PATH if kind == "product" else BENCH_LIB_PATH
        if not path.exists():
            raise FileNotFoundError(
                f"{path} is missing: build it first (python -m paper_2506_19830_amd.build or "
                "__graft_entry__.build()); the verification path has no fallback")
        lib = ctypes.CDLL(str(path))
        vp, i32p = ctypes.c_void_p, ctypes.c_void_p
        lib.la_verify_attention_workspace.restype = ctypes.c_int
        lib.la_verify_attention_workspace.argtypes = [ctypes.POINTER(la_attn_desc), ctypes.POINTER(ctypes.c_int32),
                                                      ctypes.POINTER(ctypes.c_size_t)]
        lib.la_verify_attention.restype = ctypes.c_int
        lib.la_verify_attention.argtypes = [ctypes.POINTER(la_attn_desc), vp, vp, vp, i32p, i32p,
                                            ctypes.POINTER(ctypes.c_int32), vp, vp, vp, vp, vp, vp, vp,
                                            ctypes.c_size_t, vp]
        lib.la_verify_attention_nested.restype = ctypes.c_int
        lib.la_verify_attention_nested.argtypes = [ctypes.POINTER(la_attn_desc), vp, vp, vp, i32p, i32p,
                                                   ctypes.POINTER(ctypes.c_int32), vp, vp, vp, vp, ctypes.c_int32, i32p,
                                                   ctypes.POINTER(ctypes.c_int32), vp, vp, vp, vp, vp, ctypes.c_size_t,
                                                   vp]
        lib.la_verify_attention_tree.restype = ctypes.c_int
        lib.la_verify_attention_tree.argtypes = [ctypes.POINTER(la_attn_desc), vp, vp, vp, i32p, i32p,
                                                 ctypes.POINTER(ctypes.c_int32), vp, vp, vp, vp, ctypes.c_int32, i32p,
                                                 ctypes.POINTER(ctypes.c_int32), vp, vp, vp, vp, vp, vp,
                                                 ctypes.c_size_t, vp]
        lib.la_kv_commit.restype = ctypes.c_int
        lib.la_kv_commit.argtypes = [ctypes.POINTER(la_attn_desc), vp, vp, i32p, i32p, ctypes.POINTER(ctypes.c_int32),
                                     vp, vp, vp, vp, ctypes.c_int32, i32p, i32p, i32p, vp, vp, i32p,
                                     ctypes.POINTER(la_layer_strides), vp]
        lib.la_kv_commit_tree.restype = ctypes.c_int
        lib.la_kv_commit_tree.argtypes = [ctypes.POINTER(la_attn_desc), vp, vp, i32p, i32p,
                                          ctypes.POINTER(ctypes.c_int32), vp, vp, vp, vp, ctypes.c_int32, i32p, vp,
                                          i32p, i32p, vp, vp, i32p, ctypes.POINTER(la_layer_strides), vp]
        lib.la_verify_attention_plan.restype = ctypes.c_int
        lib.la_verify_attention_plan.argtypes = [ctypes.POINTER(la_attn_desc), ctypes.POINTER(ctypes.c_int32),
                                                 ctypes.c_int32, ctypes.POINTER(la_attn_plan)]
        lib.la_step_select.restype = ctypes.c_int
        lib.la_step_select.argtypes = [ctypes.c_int32, ctypes.c_int32] + [vp] * 7
        lib.la_step_select_tree.restype = ctypes.c_int
        lib.la_step_select_tree.argtypes = [ctypes.c_int32, ctypes.c_int32] + [vp] * 7
        for fn in (lib.la_speedup_step_sync, lib.la_speedup_step_async, lib.la_speedup_token):
            fn.restype = ctypes.c_int
            fn.argtypes = [ctypes.c_double, ctypes.c_double, ctypes.c_int32, ctypes.POINTER(ctypes.c_double)]
        lib.la_plan_budget.restype = ctypes.c_int
        lib.la_plan_budget.argtypes = [ctypes.POINTER(la_plan_desc), ctypes.POINTER(ctypes.c_int32),
                                       ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)]
        lib.la_spec_accept_workspace.restype = ctypes.c_int
        lib.la_spec_accept_workspace.argtypes = [ctypes.POINTER(la_accept_desc), ctypes.POINTER(ctypes.c_size_t)]
        lib.la_spec_accept.restype = ctypes.c_int
        lib.la_spec_accept.argtypes = [ctypes.POINTER(la_accept_desc), vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                       ctypes.c_size_t, vp]
        lib.la_spec_accept_static.restype = ctypes.c_int
        lib.la_spec_accept_static.argtypes = [ctypes.POINTER(la_accept_desc)] + [vp] * 9
        lib.la_status_string.restype = ctypes.c_char_p
        lib.la_status_string.argtypes = [ctypes.c_int]
        if kind == "bench":
            lib.la_calibrate_mfma.restype = ctypes.c_int
            lib.la_calibrate_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, ctypes.POINTER(ctypes.c_double), vp]
            lib.la_calibrate_mfma_data.restype = ctypes.c_int
            lib.la_calibrate_mfma_data.argtypes = lib.la_calibrate_mfma.argtypes
            lib.la_calibrate_issue.restype = ctypes.c_int
            lib.la_calibrate_issue.argtypes = [ctypes.c_int32] * 5 + [vp, vp]
            lib.la_calibrate_read.restype = ctypes.c_int
            lib.la_calibrate_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
            lib.la_selftest_exp64.restype = ctypes.c_int
            lib.la_selftest_exp64.argtypes = [vp, vp, ctypes.c_size_t, vp]
            lib.la_check_block_tables.restype = ctypes.c_int
            lib.la_check_block_tables.argtypes = [ctypes.POINTER(la_attn_desc), vp, ctypes.POINTER(ctypes.c_int32),
                                                  ctypes.c_int32, ctypes.c_int64, vp, vp]
            lib.la_check_draft_tokens.restype = ctypes.c_int
            lib.la_check_draft_tokens.argtypes = [ctypes.POINTER(la_accept_desc), vp, vp, vp]
            lib.la_profile_enable.restype = ctypes.c_int
            lib.la_profile_enable.argtypes = [ctypes.c_int]
            lib.la_profile_select.restype = ctypes.c_int
            lib.la_profile_select.argtypes = [ctypes.c_uint32, ctypes.c_int32]
            lib.la_profile_collect.restype = ctypes.c_int
            lib.la_profile_reset.restype = ctypes.c_int
            lib.la_profile_num_kernels.restype = ctypes.c_int32
            lib.la_profile_get.restype = ctypes.c_int
            lib.la_profile_get.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_char_p),
                                           ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_double)]
        _libs[kind] = lib
    return _libs[kind]


def status_string(status: int) -> str:
    return load().la_status_string(int(status)).decode()


def _ptr(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_attn_desc(*, num_requests, num_q_heads, num_kv_heads, head_dim, gamma, branch_len, block_size,
                   max_blocks_per_request, q_dtype, kv_dtype, branch_kv_dtype, out_dtype, softmax_scale,
                   kv_split_tokens=0, kernel_shape=0) -> la_attn_desc:
    return la_attn_desc(num_requests, num_q_heads, num_kv_heads, head_dim, gamma, branch_len, block_size,
                        max_blocks_per_request, DTYPE_CODES[q_dtype], DTYPE_CODES[kv_dtype],
                        DTYPE_CODES[branch_kv_dtype], DTYPE_CODES[out_dtype], softmax_scale, kv_split_tokens,
                        kernel_shape)


def _host_lens(prefix_lens_host: Sequence[int]):
    arr = (ctypes.c_int32 * len(prefix_lens_host))(*[int(x) for x in prefix_lens_host])
    return arr


def la_verify_attention_workspace(desc: la_attn_desc, prefix_lens_host: Sequence[int]) -> int:
    out = ctypes.c_size_t(0)
    st = load().la_verify_attention_workspace(ctypes.byref(desc), _host_lens(prefix_lens_host), ctypes.byref(out))
    if st:
        raise LaError(st, "la_verify_attention_workspace")
    return int(out.value)


def la_verify_attention_plan(desc: la_attn_desc, prefix_lens_host: Sequence[int], chain_len: int = 0) -> dict:
    """What the library would launch for this problem (kernel shape, chunking, workgroups), as a dict."""
    out = la_attn_plan()
    st = load().la_verify_attention_plan(ctypes.byref(desc), _host_lens(prefix_lens_host), int(chain_len),
                                         ctypes.byref(out))
    if st:
        raise LaError(st, "la_verify_attention_plan")
    return {name: int(getattr(out, name)) for name, _ in la_attn_plan._fields_}


def la_verify_attention(desc: la_attn_desc, q, k_cache, v_cache, block_tables, prefix_lens, prefix_lens_host,
                        k_branch, v_branch, k_scale, v_scale, out, lse, workspace) -> None:
    """Enqueue one verify-attention pass on torch's current stream.  All tensors are device tensors the caller
    allocated (``workspace`` a uint8 tensor of at least ``la_verify_attention_workspace`` bytes, or None)."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load().la_verify_attention(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                    _ptr(prefix_lens), _host_lens(prefix_lens_host), _ptr(k_branch), _ptr(v_branch),
                                    _ptr(k_scale), _ptr(v_scale), _ptr(out), _ptr(lse), _ptr(workspace),
                                    ctypes.c_size_t(ws_bytes), _stream())
    if st:
        raise LaError(st, "la_verify_attention")


def la_verify_attention_nested(desc: la_attn_desc, q, k_cache, v_cache, block_tables, prefix_lens, prefix_lens_host,
                               k_branch, v_branch, k_chain, v_chain, chain_vis, chain_vis_host, k_scale, v_scale, out,
                               lse, workspace) -> None:
    """As la_verify_attention, with the drafted chain ``k_chain``/``v_chain`` [B, C, Hkv, D] and ``chain_vis``
    [B, gamma] (device int32) / ``chain_vis_host`` (nested sequence of ints, same values)."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    C = 0 if k_chain is None else int(k_chain.shape[1])
    flat = [int(x) for row in chain_vis_host for x in row] if C else []
    vis_host = (ctypes.c_int32 * max(1, len(flat)))(*flat)
    st = load().la_verify_attention_nested(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                           _ptr(block_tables), _ptr(prefix_lens), _host_lens(prefix_lens_host),
                                           _ptr(k_branch), _ptr(v_branch), _ptr(k_chain), _ptr(v_chain),
                                           ctypes.c_int32(C), _ptr(chain_vis), vis_host, _ptr(k_scale), _ptr(v_scale),
                                           _ptr(out), _ptr(lse), _ptr(workspace), ctypes.c_size_t(ws_bytes), _stream())
    if st:
        raise LaError(st, "la_verify_attention_nested")


def la_verify_attention_tree(desc: la_attn_desc, q, k_cache, v_cache, block_tables, prefix_lens, prefix_lens_host,
                             k_branch, v_branch, k_pool, v_pool, pool_seg, pool_seg_host, seg_mask, k_scale, v_scale,
                             out, lse, workspace) -> None:
    """As la_verify_attention, with the pool of drafted tokens ``k_pool``/``v_pool`` [B, C, Hkv, D], ``pool_seg``
    [B, C] (device int32; ``pool_seg_host``: nested sequence of ints, same values) and ``seg_mask`` [B, gamma]
    (device, 64-bit: torch.int64 holding the bit pattern)."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    C = 0 if k_pool is None else int(k_pool.shape[1])
    flat = [int(x) for row in pool_seg_host for x in row] if C else []
    seg_host = (ctypes.c_int32 * max(1, len(flat)))(*flat)
    st = load().la_verify_attention_tree(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                         _ptr(block_tables), _ptr(prefix_lens), _host_lens(prefix_lens_host),
                                         _ptr(k_branch), _ptr(v_branch), _ptr(k_pool), _ptr(v_pool),
                                         ctypes.c_int32(C), _ptr(pool_seg), seg_host, _ptr(seg_mask), _ptr(k_scale),
                                         _ptr(v_scale), _ptr(out), _ptr(lse), _ptr(workspace),
                                         ctypes.c_size_t(ws_bytes), _stream())
    if st:
        raise LaError(st, "la_verify_attention_tree")


def la_kv_commit(desc: la_attn_desc, k_cache, v_cache, block_tables, prefix_lens, prefix_lens_host, k_branch, v_branch,
                 k_chain, v_chain, src_branch, n_chain, n_own, k_scale, v_scale, new_prefix_lens,
                 layers: Optional[la_layer_strides] = None) -> None:
    """Append the surviving tokens' K/V to the paged cache (in place) and write the grown prefix lengths.
    ``k_chain`` may be None (no chain).  With ``layers`` the tensors hold that many layers back to back."""
    if k_chain is None:
        C = 0
    else:
        C = int(k_chain.shape[-3])   # [.., C, Hkv, D]
    st = load().la_kv_commit(ctypes.byref(desc), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables), _ptr(prefix_lens),
                             _host_lens(prefix_lens_host), _ptr(k_branch), _ptr(v_branch), _ptr(k_chain),
                             _ptr(v_chain), ctypes.c_int32(C), _ptr(src_branch), _ptr(n_chain), _ptr(n_own),
                             _ptr(k_scale), _ptr(v_scale), _ptr(new_prefix_lens),
                             ctypes.byref(layers) if layers is not None else None, _stream())
    if st:
        raise LaError(st, "la_kv_commit")


def la_kv_commit_tree(desc: la_attn_desc, k_cache, v_cache, block_tables, prefix_lens, prefix_lens_host, k_branch,
                      v_branch, k_pool, v_pool, pool_seg, commit_mask, src_branch, n_own, k_scale, v_scale,
                      new_prefix_lens, layers: Optional[la_layer_strides] = None) -> None:
    """Tree form of :func:`la_kv_commit`: the pool tokens whose node bit is set in ``commit_mask`` (int64 tensor
    holding the 64-bit masks) are appended in pool order, then ``n_own`` tokens of ``src_branch``."""
    C = 0 if k_pool is None else int(k_pool.shape[-3])
    st = load().la_kv_commit_tree(ctypes.byref(desc), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                  _ptr(prefix_lens), _host_lens(prefix_lens_host), _ptr(k_branch), _ptr(v_branch),
                                  _ptr(k_pool), _ptr(v_pool), ctypes.c_int32(C), _ptr(pool_seg), _ptr(commit_mask),
                                  _ptr(src_branch), _ptr(n_own), _ptr(k_scale), _ptr(v_scale), _ptr(new_prefix_lens),
                                  ctypes.byref(layers) if layers is not None else None, _stream())
    if st:
        raise LaError(st, "la_kv_commit_tree")


def la_calibrate_mfma(workgroups: int, iters: int, sink, data: bool = False) -> float:
    """Enqueue the pure-MFMA calibration kernel (data: on pseudo-random operands, la_calibrate_mfma_data); returns
    the launch's flop count."""
    if sink.numel() < workgroups * 512:
        raise ValueError("sink must hold workgroups * 512 floats")
    flops = ctypes.c_double()
    name = "la_calibrate_mfma_data" if data else "la_calibrate_mfma"
    st = getattr(load("bench"), name)(workgroups, iters, _ptr(sink), ctypes.byref(flops), _stream())
    if st:
        raise LaError(st, name)
    return flops.value


def la_calibrate_issue(mix: int, mix_second: int, waves: int, workgroups: int, iters: int, sink) -> None:
    """Enqueue the instruction-mix probe (see la_verify_bench.h); sink: workgroups * 512 floats."""
    st = load("bench").la_calibrate_issue(mix, mix_second, waves, workgroups, iters, _ptr(sink), _stream())
    if st:
        raise LaError(st, "la_calibrate_issue")


def la_calibrate_read(src, sink) -> int:
    """Enqueue the streaming-read calibration kernel over the whole of ``src``; returns the bytes it reads."""
    nbytes = src.numel() * src.element_size()
    st = load("bench").la_calibrate_read(_ptr(src), ctypes.c_size_t(nbytes), _ptr(sink), _stream())
    if st:
        raise LaError(st, "la_calibrate_read")
    return nbytes // 16 * 16


def la_selftest_exp64(y, out) -> None:
    """``out[i] = exp(y[i])`` as the fp64 resampling path of ``la_spec_accept`` evaluates it (device float64 tensors)."""
    st = load("bench").la_selftest_exp64(_ptr(y), _ptr(out), ctypes.c_size_t(out.numel()), _stream())
    if st:
        raise LaError(st, "la_selftest_exp64")


def la_selftest_second_attempt(on: bool) -> None:
    """Make every workgroup of the fp8 streaming shapes take its second (general-form) attempt in the calls that follow."""
    lib = load("bench")
    lib.la_selftest_second_attempt.restype = ctypes.c_int
    lib.la_selftest_second_attempt.argtypes = [ctypes.c_int]
    st = lib.la_selftest_second_attempt(int(bool(on)))
    if st:
        raise LaError(st, "la_selftest_second_attempt")


def la_check_block_tables(desc: la_attn_desc, block_tables, prefix_lens_host: Sequence[int], num_cache_blocks: int,
                          report, extra_tokens: int = 0) -> None:
    """Debug aid: count the block-table entries a call would touch that lie outside ``[0, num_cache_blocks)`` into
    ``report`` (device int32[3]: count, request, logical block of one offender)."""
    st = load("bench").la_check_block_tables(ctypes.byref(desc), _ptr(block_tables), _host_lens(prefix_lens_host),
                                             int(extra_tokens), int(num_cache_blocks), _ptr(report), _stream())
    if st:
        raise LaError(st, "la_check_block_tables")


def la_check_draft_tokens(desc: la_accept_desc, draft_tokens, report) -> None:
    """Debug aid: count the drafted token ids outside ``[0, vocab)`` into ``report`` (device int32[3]: count, branch,
    position of one offender)."""
    st = load("bench").la_check_draft_tokens(ctypes.byref(desc), _ptr(draft_tokens), _ptr(report), _stream())
    if st:
        raise LaError(st, "la_check_draft_tokens")


def la_step_select(verdicts, chain_vis, own_len):
    """Host arrays in, host arrays out: ``verdicts`` [B, nb-1] (truthy = accepted), ``chain_vis`` / ``own_len``
    [B, nb] ints.  Returns numpy int32 arrays ``(j_star, src_branch, n_chain, n_own)``, each [B]."""
    import numpy as np
    vis = np.ascontiguousarray(chain_vis, dtype=np.int32)
    own = np.ascontiguousarray(own_len, dtype=np.int32)
    nreq, nb = vis.shape
    v = np.ascontiguousarray(np.asarray(verdicts, dtype=bool).reshape(nreq, nb - 1), dtype=np.uint8)
    outs = [np.empty(nreq, dtype=np.int32) for _ in range(4)]
    st = load().la_step_select(nreq, nb, v.ctypes.data if v.size else None, vis.ctypes.data, own.ctypes.data,
                               *(o.ctypes.data for o in outs))
    if st:
        raise LaError(st, "la_step_select")
    return tuple(outs)


def la_step_select_tree(parent, verdicts, own_len):
    """Host arrays: ``parent`` [nodes] (-1 = child of the root), ``verdicts`` [B, nodes] (truthy = accepted),
    ``own_len`` [B, nodes + 1].  Returns ``(depth, commit_mask, src_branch, n_own)``: int32 [B], uint64 [B],
    int32 [B], int32 [B]."""
    import numpy as np
    par = np.ascontiguousarray(parent, dtype=np.int32)
    own = np.ascontiguousarray(own_len, dtype=np.int32)
    nreq, nodes = own.shape[0], par.shape[0]
    if own.shape[1] != nodes + 1:
        raise ValueError("own_len must be [B, nodes + 1]")
    v = np.ascontiguousarray(np.asarray(verdicts, dtype=bool).reshape(nreq, nodes), dtype=np.uint8)
    depth, src, n_own = (np.empty(nreq, dtype=np.int32) for _ in range(3))
    mask = np.empty(nreq, dtype=np.uint64)
    st = load().la_step_select_tree(nreq, nodes, par.ctypes.data if nodes else None, v.ctypes.data if nodes else None,
                                    own.ctypes.data, depth.ctypes.data, mask.ctypes.data, src.ctypes.data,
                                    n_own.ctypes.data)
    if st:
        raise LaError(st, "la_step_select_tree")
    return depth, mask, src, n_own


def _speedup(fn_name: str, alpha: float, c: float, k: int) -> float:
    out = ctypes.c_double()
    st = getattr(load(), fn_name)(alpha, c, k, ctypes.byref(out))
    if st:
        raise LaError(st, fn_name)
    return out.value


def la_speedup_step_sync(alpha1: float, c1: float, k1: int) -> float:
    return _speedup("la_speedup_step_sync", alpha1, c1, k1)


def la_speedup_step_async(alpha1: float, c1: float, k1: int) -> float:
    return _speedup("la_speedup_step_async", alpha1, c1, k1)


def la_speedup_token(alpha2: float, c2: float, k2: int) -> float:
    return _speedup("la_speedup_token", alpha2, c2, k2)


def la_plan_budget(alpha1: float, c1: float, alpha2: float, c2: float, budget: int, asynchronous: bool):
    """Returns ``(k1, k2, speedup)``."""
    d = la_plan_desc(alpha1, c1, alpha2, c2, budget, 1 if asynchronous else 0)
    k1, k2, h = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_double()
    st = load().la_plan_budget(ctypes.byref(d), ctypes.byref(k1), ctypes.byref(k2), ctypes.byref(h))
    if st:
        raise LaError(st, "la_plan_budget")
    return k1.value, k2.value, h.value


def make_accept_desc(*, num_branches, num_draft, vocab, logits_dtype, temperature=1.0, top_k=0,
                     top_p=1.0) -> la_accept_desc:
    return la_accept_desc(num_branches, num_draft, vocab, DTYPE_CODES[logits_dtype], temperature, top_k, top_p)


def la_spec_accept_workspace(desc: la_accept_desc) -> int:
    out = ctypes.c_size_t(0)
    st = load().la_spec_accept_workspace(ctypes.byref(desc), ctypes.byref(out))
    if st:
        raise LaError(st, "la_spec_accept_workspace")
    return int(out.value)


def la_spec_accept(desc: la_accept_desc, target_logits, draft_logits, draft_tokens, u_accept, u_sample,
                   accepted_len, next_token, accept_ratio, workspace) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load().la_spec_accept(ctypes.byref(desc), _ptr(target_logits), _ptr(draft_logits), _ptr(draft_tokens),
                               _ptr(u_accept), _ptr(u_sample), _ptr(accepted_len), _ptr(next_token),
                               _ptr(accept_ratio), _ptr(workspace), ctypes.c_size_t(ws_bytes), _stream())
    if st:
        raise LaError(st, "la_spec_accept")


def la_spec_accept_static(desc: la_accept_desc, target_logits, draft_logits, draft_tokens, u_accept, u_sample,
                          accepted_len, next_token, accept_ratio) -> None:
    """``la_spec_accept`` on the library's own scratch array (no workspace, nothing allocated)."""
    st = load().la_spec_accept_static(ctypes.byref(desc), _ptr(target_logits), _ptr(draft_logits),
                                      _ptr(draft_tokens), _ptr(u_accept), _ptr(u_sample), _ptr(accepted_len),
                                      _ptr(next_token), _ptr(accept_ratio), _stream())
    if st:
        raise LaError(st, "la_spec_accept_static")


# ------------------------------------------------------------------------------------------- profiling

def la_profile_enable(on: bool) -> None:
    load("bench").la_profile_enable(int(bool(on)))


def la_profile_select(kernels=None, stride: int = 1) -> None:
    """Time only the named kernels (None = all), and of their launches every ``stride``-th one."""
    lib = load("bench")
    mask = 0xFFFFFFFF
    if kernels is not None:
        names = {}
        for slot in range(lib.la_profile_num_kernels()):
            name = ctypes.c_char_p()
            lib.la_profile_get(slot, ctypes.byref(name), ctypes.byref(ctypes.c_int64()), ctypes.byref(ctypes.c_double()))
            names[name.value.decode()] = slot
        mask = 0
        for k in kernels:
            mask |= 1 << names[k]
    st = lib.la_profile_select(mask, int(stride))
    if st:
        raise LaError(st, "la_profile_select")


def la_profile_reset() -> None:
    load("bench").la_profile_reset()


def la_profile_collect() -> dict:
    """Synchronise on the recorded events; returns {kernel: (launches, total_ms)} since the last reset."""
    lib = load("bench")
    st = lib.la_profile_collect()
    if st:
        raise LaError(st, "la_profile_collect")
    res = {}
    for slot in range(lib.la_profile_num_kernels()):
        name = ctypes.c_char_p()
        n = ctypes.c_int64()
        ms = ctypes.c_double()
        lib.la_profile_get(slot, ctypes.byref(name), ctypes.byref(n), ctypes.byref(ms))
        res[name.value.decode()] = (int(n.value), float(ms.value))
    return res


# ------------------------------------------------------------------------------------------- tensor plumbing

def to_device(bits, dtype: str, device="cuda") -> Optional[torch.Tensor]:
    """numpy storage array (fp32 / uint16 bf16 bits / uint8 fp8 bits) -> device tensor of the matching torch dtype."""
    if bits is None:
        return None
    import numpy as np
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(bits, dtype=np.float32)).to(device)
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)
    if dtype == "fp8_e4m3":
        return torch.from_numpy(np.ascontiguousarray(bits)).to(device).view(torch.float8_e4m3fn)
    raise ValueError(dtype)


def empty_out(shape, dtype: str, device="cuda") -> torch.Tensor:
    return torch.empty(shape, dtype=_TORCH_DTYPES[dtype], device=device)
