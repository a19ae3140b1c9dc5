"""ctypes front end of the fp64 CPU oracle (``la_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this module;
it exists so that tests, the smoke check and the benchmark's CPU-baseline leg
can evaluate the plain definition of the verification pass (Section 3.1 /
Algorithm 1 for the attention over "prefix ++ own branch", Section 2 for the
token-level accept/resample rule) on the same bytes the GPU receives.

Arrays are numpy; bf16 tensors travel as ``uint16`` bit patterns and fp8-e4m3fn
tensors as ``uint8`` bit patterns, because numpy has neither type.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "la_oracle.c"
_LIB = _HERE / "libla_oracle.so"

DTYPE_CODES = {"f32": 0, "bf16": 1, "fp8_e4m3": 2, "f64": 3}
_NP_STORAGE = {"f32": np.float32, "bf16": np.uint16, "fp8_e4m3": np.uint8, "f64": np.float64}


def build(force: bool = False) -> Path:
    """Compile ``la_oracle.c`` with gcc (fp64, no fast-math, no FMA contraction)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        cmd = ["gcc", "-O2", "-ftree-vectorize", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", str(tmp), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitized(out: Path) -> Path:
    """``la_oracle.c`` with gcc's address and undefined-behaviour sanitizers, for the test that runs the pins
    under them (load it with ``LA_ORACLE_LIB`` and gcc's libasan preloaded)."""
    cmd = ["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", str(out), str(_SRC), "-lm"]
    subprocess.run(cmd, check=True)
    return out


_lib = None


def _load():
    global _lib
    if _lib is None:
        override = os.environ.get("LA_ORACLE_LIB")   # used by the mutation test to load a deliberately broken build
        _lib = ctypes.CDLL(override if override else str(build()))
        _lib.lao_verify_attention.restype = ctypes.c_int
        _lib.lao_verify_attention_nested.restype = ctypes.c_int
        _lib.lao_verify_attention_tree.restype = ctypes.c_int
        _lib.lao_attention_row_weights.restype = ctypes.c_int
        _lib.lao_spec_accept.restype = ctypes.c_int
        _lib.lao_spec_accept_warped.restype = ctypes.c_int
        _lib.lao_warp_probs.restype = ctypes.c_int
        _lib.lao_widen.restype = ctypes.c_int
        _lib.lao_kv_commit.restype = ctypes.c_int
        _lib.lao_kv_commit_tree.restype = ctypes.c_int
        _lib.lao_quantize_fp8_e4m3.restype = ctypes.c_int
        _lib.lao_num_threads.restype = ctypes.c_int
    return _lib


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else ctypes.c_void_p(0)


def _storage(a, dtype: str, name: str):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype != _NP_STORAGE[dtype]:
        raise TypeError(f"{name}: dtype {dtype} must be stored as {_NP_STORAGE[dtype].__name__}, got {a.dtype}")
    return a


def num_threads() -> int:
    return int(_load().lao_num_threads())


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact fp64 value of every stored element."""
    bits = _storage(bits, dtype, "bits")
    out = np.empty(bits.shape, dtype=np.float64)
    rc = _load().lao_widen(_ptr(bits), DTYPE_CODES[dtype], ctypes.c_int64(bits.size), _ptr(out))
    if rc:
        raise ValueError("lao_widen rejected its arguments")
    return out


def _attn_args(q, k_cache, v_cache, block_tables, prefix_lens, k_branch, v_branch, k_scale, v_scale, *, q_dtype,
               kv_dtype, branch_kv_dtype, block_size, scale):
    q = _storage(q, q_dtype, "q")
    k_branch = _storage(k_branch, branch_kv_dtype, "k_branch")
    v_branch = _storage(v_branch, branch_kv_dtype, "v_branch")
    k_cache = _storage(k_cache, kv_dtype, "k_cache")
    v_cache = _storage(v_cache, kv_dtype, "v_cache")
    B, gamma, L, Hq, D = q.shape
    Hkv = k_branch.shape[3]
    if k_branch.shape != (B, gamma, L, Hkv, D) or v_branch.shape != k_branch.shape:
        raise ValueError("branch K/V shape mismatch")
    prefix_lens = np.ascontiguousarray(prefix_lens, dtype=np.int32)
    if prefix_lens.shape != (B,):
        raise ValueError("prefix_lens must be [B]")
    if block_tables is not None:
        block_tables = np.ascontiguousarray(block_tables, dtype=np.int32)
        max_blocks = block_tables.shape[1]
        if block_tables.shape[0] != B:
            raise ValueError("block_tables must be [B, max_blocks]")
        if k_cache is not None and block_tables.size and int(block_tables.max()) >= k_cache.shape[0]:
            raise ValueError("block id out of range")
    else:
        if k_cache is None:
            max_blocks = 0
        else:
            if k_cache.shape[0] % B:
                raise ValueError("identity mapping needs num_blocks divisible by B")
            max_blocks = k_cache.shape[0] // B
    if k_cache is not None:
        if k_cache.shape[1:] != (Hkv, block_size, D) or v_cache.shape != k_cache.shape:
            raise ValueError("cache must be [num_blocks, Hkv, block_size, D]")
    if k_scale is not None:
        k_scale = np.ascontiguousarray(k_scale, dtype=np.float32)
        v_scale = np.ascontiguousarray(v_scale, dtype=np.float32)
        if k_scale.shape != (Hkv,) or v_scale.shape != (Hkv,):
            raise ValueError("scales must be [Hkv]")
    keep = (q, k_cache, v_cache, block_tables, prefix_lens, k_branch, v_branch, k_scale, v_scale)
    head = (ctypes.c_int(B), ctypes.c_int(gamma), ctypes.c_int(L), ctypes.c_int(Hq), ctypes.c_int(Hkv),
            ctypes.c_int(D), ctypes.c_int(block_size), ctypes.c_int(max_blocks), ctypes.c_int(DTYPE_CODES[q_dtype]),
            ctypes.c_int(DTYPE_CODES[kv_dtype]), ctypes.c_int(DTYPE_CODES[branch_kv_dtype]), ctypes.c_double(scale),
            _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables), _ptr(prefix_lens), _ptr(k_branch),
            _ptr(v_branch), _ptr(k_scale), _ptr(v_scale))
    return head, keep, (B, gamma, L, Hq, D)


def verify_attention(q, k_cache, v_cache, block_tables, prefix_lens, k_branch, v_branch, k_scale=None, v_scale=None,
                     *, q_dtype, kv_dtype, branch_kv_dtype, block_size, scale, row_ids=None, k_chain=None,
                     v_chain=None, chain_vis=None, k_pool=None, v_pool=None, pool_seg=None, seg_mask=None):
    """Attention of every branch token over ``prefix ++ own branch`` (causal inside the branch).  Nested form:
    with ``k_chain``/``v_chain`` ``[B, C, Hkv, D]`` (branch storage dtype) and ``chain_vis`` ``[B, gamma]``, branch g
    sees ``prefix ++ chain[:chain_vis[b, g]] ++ own branch``.  Tree form: with ``k_pool``/``v_pool``
    ``[B, C, Hkv, D]``, ``pool_seg`` ``[B, C]`` (segment 0..63 of every pool token) and ``seg_mask`` ``[B, gamma]``
    (uint64), branch g sees the pool tokens whose segment bit is set in its mask, in pool order.

    Returns ``(out, lse)`` in fp64.  Without ``row_ids`` the shapes are
    ``[B, gamma, L, Hq, D]`` and ``[B, gamma, L, Hq]``; with ``row_ids`` (flat
    ids ``((b*gamma+g)*L+i)*Hq+h``) they are ``[n, D]`` and ``[n]``.
    """
    head, keep, (B, gamma, L, Hq, D) = _attn_args(q, k_cache, v_cache, block_tables, prefix_lens, k_branch, v_branch,
                                                   k_scale, v_scale, q_dtype=q_dtype, kv_dtype=kv_dtype,
                                                   branch_kv_dtype=branch_kv_dtype, block_size=block_size,
                                                   scale=scale)
    if row_ids is None:
        n = B * gamma * L * Hq
        ids = None
        out = np.empty((B, gamma, L, Hq, D), dtype=np.float64)
        lse = np.empty((B, gamma, L, Hq), dtype=np.float64)
    else:
        ids = np.ascontiguousarray(row_ids, dtype=np.int64)
        n = ids.size
        out = np.empty((n, D), dtype=np.float64)
        lse = np.empty((n,), dtype=np.float64)
    if k_pool is not None:
        if k_chain is not None:
            raise ValueError("give a chain or a pool, not both")
        kp = _storage(k_pool, branch_kv_dtype, "k_pool")
        vp = _storage(v_pool, branch_kv_dtype, "v_pool")
        C = kp.shape[1]
        seg = np.ascontiguousarray(pool_seg, dtype=np.int32)
        mask = np.ascontiguousarray(seg_mask, dtype=np.uint64)
        if seg.shape != (B, C) or mask.shape != (B, gamma) or kp.shape != vp.shape or kp.shape[0] != B or \
                kp.shape[3] != D:
            raise ValueError("k_pool/v_pool must be [B, C, Hkv, D], pool_seg [B, C], seg_mask [B, gamma]")
        rc = _load().lao_verify_attention_tree(*head, ctypes.c_int(C), _ptr(kp), _ptr(vp), _ptr(seg), _ptr(mask),
                                               _ptr(ids), ctypes.c_int64(n), _ptr(out), _ptr(lse))
        del keep
        if rc:
            raise ValueError("lao_verify_attention_tree rejected its arguments")
        return out, lse
    if k_chain is None:
        C, kc, vc, vis = 0, None, None, None
    else:
        kc = _storage(k_chain, branch_kv_dtype, "k_chain")
        vc = _storage(v_chain, branch_kv_dtype, "v_chain")
        C = kc.shape[1]
        vis = np.ascontiguousarray(chain_vis, dtype=np.int32)
        if vis.shape != (B, gamma) or kc.shape != vc.shape or kc.shape[0] != B or kc.shape[3] != D:
            raise ValueError("k_chain/v_chain must be [B, C, Hkv, D] and chain_vis [B, gamma]")
    rc = _load().lao_verify_attention_nested(*head, ctypes.c_int(C), _ptr(kc), _ptr(vc), _ptr(vis), _ptr(ids),
                                             ctypes.c_int64(n), _ptr(out), _ptr(lse))
    del keep
    if rc:
        raise ValueError("lao_verify_attention rejected its arguments")
    return out, lse


def attention_row_weights(q, k_cache, v_cache, block_tables, prefix_lens, k_branch, v_branch, k_scale=None,
                          v_scale=None, *, q_dtype, kv_dtype, branch_kv_dtype, block_size, scale, row_id):
    """Softmax weights of one query row over its visible keys (prefix, then branch tokens 0..i)."""
    head, keep, (B, gamma, L, Hq, D) = _attn_args(q, k_cache, v_cache, block_tables, prefix_lens, k_branch, v_branch,
                                                   k_scale, v_scale, q_dtype=q_dtype, kv_dtype=kv_dtype,
                                                   branch_kv_dtype=branch_kv_dtype, block_size=block_size,
                                                   scale=scale)
    i = (row_id // Hq) % L
    b = row_id // Hq // L // gamma
    w = np.empty((int(keep[4][b]) + i + 1,), dtype=np.float64)
    rc = _load().lao_attention_row_weights(*head, ctypes.c_int64(row_id), _ptr(w))
    del keep
    if rc:
        raise ValueError("lao_attention_row_weights rejected its arguments")
    return w


def _commit_operands(k_cache, v_cache, block_tables, prefix_lens, k_branch, v_branch, k_drafted, v_drafted, k_scale,
                     v_scale, kv_dtype, branch_kv_dtype, block_size):
    """Argument marshalling shared by the two commit wrappers (no arithmetic)."""
    kc = _storage(k_cache, kv_dtype, "k_cache").copy()
    vc = _storage(v_cache, kv_dtype, "v_cache").copy()
    kb = _storage(k_branch, branch_kv_dtype, "k_branch")
    vb = _storage(v_branch, branch_kv_dtype, "v_branch")
    B, gamma, L, Hkv, D = kb.shape
    lens = np.ascontiguousarray(prefix_lens, dtype=np.int32)
    if block_tables is not None:
        block_tables = np.ascontiguousarray(block_tables, dtype=np.int32)
        max_blocks = block_tables.shape[1]
        if int(block_tables.max()) >= kc.shape[0]:
            raise ValueError("block id out of range")
    else:
        max_blocks = kc.shape[0] // B
    if kc.shape[1:] != (Hkv, block_size, D) or vc.shape != kc.shape:
        raise ValueError("cache must be [num_blocks, Hkv, block_size, D]")
    if k_drafted is None:
        C, kd, vd = 0, None, None
    else:
        kd = _storage(k_drafted, branch_kv_dtype, "k_chain")
        vd = _storage(v_drafted, branch_kv_dtype, "v_chain")
        C = kd.shape[1]
        if kd.shape != (B, C, Hkv, D) or vd.shape != kd.shape:
            raise ValueError("drafted K/V must be [B, C, Hkv, D]")
    ks = None if k_scale is None else np.ascontiguousarray(k_scale, dtype=np.float32)
    vs = None if v_scale is None else np.ascontiguousarray(v_scale, dtype=np.float32)
    shape = [ctypes.c_int(x) for x in (B, gamma, L, Hkv, D, block_size, max_blocks, DTYPE_CODES[kv_dtype],
                                       DTYPE_CODES[branch_kv_dtype])]
    return shape, kc, vc, block_tables, lens, kb, vb, C, kd, vd, ks, vs


def kv_commit(k_cache, v_cache, block_tables, prefix_lens, k_branch, v_branch, k_chain, v_chain, src_branch, n_chain,
              n_own, k_scale=None, v_scale=None, *, kv_dtype, branch_kv_dtype, block_size):
    """Append, per request, the first ``n_chain[b]`` tokens of the drafted chain and then the first ``n_own[b]``
    tokens of branch ``src_branch[b]`` behind the prefix (Algorithm 1, once j* is known).

    Returns ``(k_cache, v_cache, new_prefix_lens)``: updated *copies* of the caches (storage bit patterns) and the
    grown prefix lengths.  ``k_chain`` may be ``None`` (no chain: ``n_chain`` must be all zero)."""
    shape, kc, vc, tables, lens, kb, vb, C, kch, vch, ks, vs = _commit_operands(
        k_cache, v_cache, block_tables, prefix_lens, k_branch, v_branch, k_chain, v_chain, k_scale, v_scale, kv_dtype,
        branch_kv_dtype, block_size)
    sb = np.ascontiguousarray(src_branch, dtype=np.int32)
    nc = np.ascontiguousarray(n_chain, dtype=np.int32)
    no = np.ascontiguousarray(n_own, dtype=np.int32)
    new_lens = np.empty(lens.shape, dtype=np.int32)
    rc = _load().lao_kv_commit(*shape, _ptr(kc), _ptr(vc), _ptr(tables), _ptr(lens), _ptr(kb), _ptr(vb),
                               ctypes.c_int(C), _ptr(kch), _ptr(vch), _ptr(sb), _ptr(nc), _ptr(no), _ptr(ks),
                               _ptr(vs), _ptr(new_lens))
    if rc:
        raise ValueError(f"lao_kv_commit rejected its arguments (status {rc})")
    return kc, vc, new_lens


def kv_commit_tree(k_cache, v_cache, block_tables, prefix_lens, k_branch, v_branch, k_pool, v_pool, pool_seg,
                   commit_mask, src_branch, n_own, k_scale=None, v_scale=None, *, kv_dtype, branch_kv_dtype,
                   block_size):
    """Tree form of :func:`kv_commit` (Section 3.1, "Multi-Branch Drafting"): the pool tokens whose node
    (``pool_seg[b][c]``) has its bit set in ``commit_mask[b]`` are appended in pool order, then the first
    ``n_own[b]`` tokens of branch ``src_branch[b]``."""
    shape, kc, vc, tables, lens, kb, vb, C, kp, vp, ks, vs = _commit_operands(
        k_cache, v_cache, block_tables, prefix_lens, k_branch, v_branch, k_pool, v_pool, k_scale, v_scale, kv_dtype,
        branch_kv_dtype, block_size)
    seg = None if pool_seg is None else np.ascontiguousarray(pool_seg, dtype=np.int32)
    if C and (seg is None or seg.shape != (lens.shape[0], C)):
        raise ValueError("pool_seg must be [B, C]")
    cm = np.ascontiguousarray(commit_mask, dtype=np.uint64)
    sb = np.ascontiguousarray(src_branch, dtype=np.int32)
    no = np.ascontiguousarray(n_own, dtype=np.int32)
    new_lens = np.empty(lens.shape, dtype=np.int32)
    rc = _load().lao_kv_commit_tree(*shape, _ptr(kc), _ptr(vc), _ptr(tables), _ptr(lens), _ptr(kb), _ptr(vb),
                                    ctypes.c_int(C), _ptr(kp), _ptr(vp), _ptr(seg), _ptr(cm), _ptr(sb), _ptr(no),
                                    _ptr(ks), _ptr(vs), _ptr(new_lens))
    if rc:
        raise ValueError(f"lao_kv_commit_tree rejected its arguments (status {rc})")
    return kc, vc, new_lens


def quantize_fp8_e4m3(x, scale: float) -> np.ndarray:
    """Test hook: e4m3fn codes of ``x / scale`` (fp32 quotient, nearest, ties to even, saturating)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint8)
    rc = _load().lao_quantize_fp8_e4m3(_ptr(x), ctypes.c_int64(x.size), ctypes.c_float(scale), _ptr(out))
    if rc:
        raise ValueError("lao_quantize_fp8_e4m3 rejected its arguments")
    return out


def warp_probs(logits, *, logits_dtype, temperature=1.0, top_k=0, top_p=1.0):
    """Test hook: the target distribution of one logit row [V] after temperature, top-k and top-p.
    Returns (p [V] fp64, margin) with margin the closest relative distance of a top-p decision to its threshold."""
    a = _storage(logits, logits_dtype, "logits")
    V = a.shape[-1]
    out = np.empty((V,), dtype=np.float64)
    mg = ctypes.c_double(0.0)
    rc = _load().lao_warp_probs(_ptr(a), ctypes.c_int(DTYPE_CODES[logits_dtype]), ctypes.c_int(V),
                                ctypes.c_double(temperature), ctypes.c_int(top_k), ctypes.c_double(top_p), _ptr(out),
                                ctypes.byref(mg))
    if rc:
        raise ValueError("lao_warp_probs rejected its arguments")
    return out, float(mg.value)


def spec_accept(target_logits, draft_logits, draft_tokens, u_accept, u_sample, *, logits_dtype, temperature=1.0,
                top_k=0, top_p=1.0):
    """Sequential token-level accept / resample.  Returns a dict with
    ``accepted_len`` [NB], ``next_token`` [NB], ``ratio`` [NB,K], ``margin`` [NB,K],
    ``cdf_lo`` [NB], ``cdf_hi`` [NB], ``warp_margin`` [NB].  ``draft_logits=None``: point-mass draft at the
    drafted tokens.  ``top_k`` (0 = off) / ``top_p`` (1 = off) warp the target distribution."""
    t = _storage(target_logits, logits_dtype, "target_logits")
    d = None if draft_logits is None else _storage(draft_logits, logits_dtype, "draft_logits")
    NB, K1, V = t.shape
    K = K1 - 1
    if d is not None and d.shape != (NB, K, V):
        raise ValueError("draft_logits must be [NB, K, V] with target_logits [NB, K+1, V]")
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    ua = np.ascontiguousarray(u_accept, dtype=np.float32)
    us = np.ascontiguousarray(u_sample, dtype=np.float32)
    if tok.shape != (NB, K) or ua.shape != (NB, K) or us.shape != (NB,):
        raise ValueError("draft_tokens/u_accept must be [NB, K], u_sample [NB]")
    n = np.empty((NB,), dtype=np.int32)
    nxt = np.empty((NB,), dtype=np.int32)
    ratio = np.empty((NB, K), dtype=np.float64)
    margin = np.empty((NB, K), dtype=np.float64)
    lo = np.empty((NB,), dtype=np.float64)
    hi = np.empty((NB,), dtype=np.float64)
    wm = np.empty((NB,), dtype=np.float64)
    rc = _load().lao_spec_accept_warped(ctypes.c_int(NB), ctypes.c_int(K), ctypes.c_int(V),
                                        ctypes.c_int(DTYPE_CODES[logits_dtype]), ctypes.c_double(temperature),
                                        ctypes.c_int(top_k), ctypes.c_double(top_p), _ptr(t), _ptr(d), _ptr(tok),
                                        _ptr(ua), _ptr(us), _ptr(n), _ptr(nxt), _ptr(ratio), _ptr(margin), _ptr(lo),
                                        _ptr(hi), _ptr(wm))
    if rc:
        raise ValueError("lao_spec_accept rejected its arguments")
    return {"accepted_len": n, "next_token": nxt, "ratio": ratio, "margin": margin, "cdf_lo": lo, "cdf_hi": hi,
            "warp_margin": wm}
