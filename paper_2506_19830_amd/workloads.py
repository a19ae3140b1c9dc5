"""Seeded synthetic inputs shaped like the paper's workloads.

This module only *produces inputs* (random tensors, storage-format encoding,
block tables, drafted tokens).  It holds none of the arithmetic of the
verification pass itself, so both the HIP path and the CPU checker can be fed
from it without sharing any of the method's code.

The paper evaluates 32B-class GQA reasoning models (Section 4, "Models" and
"General Parameters": generations of up to 32K/37K tokens, a handful of
drafted steps verified per pass, 8 speculative tokens for token-level SD).  Its
weights and datasets are not available here, so every case below is random
data of those shapes; the five numbered cases are the benchmark
configurations this repository is measured on.

bf16 tensors are returned as ``uint16`` bit patterns and fp8-e4m3fn tensors as
``uint8`` bit patterns (numpy has neither type).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, Optional, Tuple

import numpy as np

FP8_E4M3_MAX = 448.0


# ----------------------------------------------------------------------------- storage encoders

def encode_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def _fp8_positive_values() -> np.ndarray:
    vals = []
    for code in range(127):  # 0x00 .. 0x7E, 0x7F is NaN
        e, m = code >> 3, code & 7
        vals.append((m / 8.0) * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7))
    return np.asarray(vals, dtype=np.float64)


_FP8_VALUES = _fp8_positive_values()


def encode_fp8_e4m3(x: np.ndarray) -> np.ndarray:
    """fp32 -> OCP e4m3fn bit patterns: round to nearest even, saturate at +-448."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    a = np.minimum(np.abs(x).astype(np.float64), FP8_E4M3_MAX)
    lo = np.searchsorted(_FP8_VALUES, a, side="right") - 1
    hi = np.minimum(lo + 1, 126)
    d_lo = a - _FP8_VALUES[lo]
    d_hi = _FP8_VALUES[hi] - a
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (lo % 2 == 1))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    return code | (np.signbit(x).astype(np.uint8) << np.uint8(7))


def encode(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return encode_bf16(x)
    if dtype == "fp8_e4m3":
        return encode_fp8_e4m3(x)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------- case descriptions

@dataclass(frozen=True)
class AttnCase:
    """One verify-attention workload: B requests, gamma branches of L tokens each."""
    name: str
    prefix_lens: Tuple[int, ...]
    gamma: int
    L: int
    Hq: int
    Hkv: int
    D: int
    q_dtype: str = "bf16"
    kv_dtype: str = "bf16"
    branch_kv_dtype: str = "bf16"
    out_dtype: str = "bf16"
    block_size: int = 16
    paged: bool = False          # random block table over a shared pool
    seed: int = 0
    layer: int = 0               # stream offset so that layers of a sweep differ
    spare_tokens: int = 0        # cache room (mapped by the block table) behind every prefix, for the KV commit
    late_key_shift: float = 0.0  # nats by which every score against a key from token `late_from` on (branch keys
    late_from: int = 64          # included) lies above N(0,1): a running maximum that jumps far, late in the prefix

    @property
    def B(self) -> int:
        return len(self.prefix_lens)

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)

    @property
    def max_blocks(self) -> int:
        return max(1, max(-(-(p + self.spare_tokens) // self.block_size) for p in self.prefix_lens))

    @property
    def branch_tokens(self) -> int:
        return self.B * self.gamma * self.L

    def flops(self) -> float:
        """4*D flops per (query row, visible key) pair."""
        per_req = [self.gamma * self.L * self.Hq * 4.0 * self.D * (p + (self.L + 1) / 2.0) for p in self.prefix_lens]
        return float(sum(per_req))

    def algorithmic_bytes(self) -> float:
        """Every K/V/Q element read once, every output element written once."""
        sz = {"f32": 4, "bf16": 2, "fp8_e4m3": 1}
        kv = sum(2 * self.Hkv * p * self.D * sz[self.kv_dtype] for p in self.prefix_lens)
        rows = self.branch_tokens
        br = 2 * rows * self.Hkv * self.D * sz[self.branch_kv_dtype]
        qo = rows * self.Hq * self.D * (sz[self.q_dtype] + sz[self.out_dtype])
        return float(kv + br + qo)


@dataclass(frozen=True)
class AcceptCase:
    """One accept/resample workload: NB branches, K drafted tokens each, vocabulary V."""
    name: str
    NB: int
    K: int
    V: int
    logits_dtype: str = "bf16"
    target_std: float = 3.0
    draft_noise_std: Optional[float] = 1.0   # draft = target + N(0, noise^2); None => independent N(0, target_std^2)
    temperature: float = 1.0
    seed: int = 0
    top_k: int = 0                # 0 = off
    top_p: float = 1.0            # 1 = off; an fp32 field of the descriptor: checkers must use float(np.float32(top_p))
    point_mass: bool = False      # the drafter gives tokens only (prompt-lookup drafts): no draft logits
    peak: float = 16.0            # point_mass: added to the target logit of every drafted token, so that p(x) is O(0.1..1)

    def algorithmic_bytes(self) -> float:
        sz = {"f32": 4, "bf16": 2}[self.logits_dtype]
        rows = (self.K + 1) if self.point_mass else (2 * self.K + 1)
        return float(self.NB * rows * self.V * sz)


def config(n: int) -> Tuple[AttnCase, AcceptCase]:
    """The five benchmark configurations (1-based)."""
    if n == 1:
        return (AttnCase("cfg1_tiny_f32", (256,), 2, 8, 4, 1, 64, "f32", "f32", "f32", "f32"),
                AcceptCase("cfg1_accept", 2, 4, 512, "f32", target_std=2.0, draft_noise_std=None))
    if n == 2:
        return (AttnCase("cfg2_p4k_g4x32", (4096,), 4, 32, 64, 8, 128),
                AcceptCase("cfg2_accept", 4, 4, 152064, "bf16"))
    if n == 3:
        return (AttnCase("cfg3_p16k_g8x64", (16384,), 8, 64, 40, 8, 128),
                AcceptCase("cfg3_accept", 8, 8, 152064, "f32"))
    if n == 4:
        return (AttnCase("cfg4_paged_4req", (8192, 16384, 24576, 32768), 8, 48, 64, 8, 128, paged=True),
                AcceptCase("cfg4_accept", 32, 8, 152064, "bf16"))
    if n == 5:
        return (AttnCase("cfg5_p32k_g8x64_fp8", (32768,), 8, 64, 40, 8, 128, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16"),
                AcceptCase("cfg5_accept", 8, 8, 152064, "bf16"))
    if n == 6:
        # not one of the benchmark's five: the operating point of the paper's own runs (Section 4, General
        # Parameters: 6 speculative steps verified together, each target pass carrying 1 + 8 tokens per branch under
        # prompt-lookup drafting, temperature 0.6 / top-p 0.95), at configuration 5's model shape and cache
        return (AttnCase("paper_step_p32k_g6x9_fp8", (32768,), 6, 9, 40, 8, 128, "bf16", "fp8_e4m3", "fp8_e4m3",
                         "bf16"),
                AcceptCase("paper_step_accept", 6, 8, 152064, "bf16", temperature=0.6, top_p=0.95, point_mass=True,
                           peak=9.0))
    raise ValueError("configs are numbered 1..5 (6: the paper's own operating point)")


NUM_LAYERS_CFG5 = 64


# ----------------------------------------------------------------------------- numpy generators

def _rng(seed: int, stream: int) -> np.random.Generator:
    # Philox is counter based: (seed, stream) names an independent sequence.
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, stream]))


def make_attention_inputs(case: AttnCase) -> Dict[str, Optional[np.ndarray]]:
    """Q/K/V ~ N(0,1) in the case's storage types, plus cache layout metadata.

    cache layout  [num_blocks, Hkv, block_size, D]; branch tensors [B, gamma, L, H, D].
    Contiguous cases own ``max_blocks`` consecutive blocks per request and pass
    ``block_tables=None``; paged cases draw a random permutation of a pool that
    holds exactly the blocks needed.  fp8 caches carry one scale per KV head
    (amax/448); a branch K/V stored as fp8 reuses the cache's scales.
    """
    c = case
    s0 = 16 * c.layer
    B, bs = c.B, c.block_size
    blocks_needed = [-(-(p + c.spare_tokens) // bs) for p in c.prefix_lens]
    if c.paged:
        num_blocks = max(1, sum(blocks_needed))
        perm = _rng(c.seed, s0 + 7).permutation(num_blocks).astype(np.int32)
        tables = np.zeros((B, c.max_blocks), dtype=np.int32)
        at = 0
        for b, nb in enumerate(blocks_needed):
            tables[b, :nb] = perm[at:at + nb]
            at += nb
    else:
        num_blocks = B * c.max_blocks
        tables = None

    q = _rng(c.seed, s0 + 0).standard_normal((B, c.gamma, c.L, c.Hq, c.D), dtype=np.float32)
    kb = _rng(c.seed, s0 + 1).standard_normal((B, c.gamma, c.L, c.Hkv, c.D), dtype=np.float32)
    vb = _rng(c.seed, s0 + 2).standard_normal((B, c.gamma, c.L, c.Hkv, c.D), dtype=np.float32)
    kc = _rng(c.seed, s0 + 3).standard_normal((num_blocks, c.Hkv, bs, c.D), dtype=np.float32)
    vc = _rng(c.seed, s0 + 4).standard_normal((num_blocks, c.Hkv, bs, c.D), dtype=np.float32)

    if c.late_key_shift != 0.0:
        # a +-1 direction u per KV head, added to every query (of the head's group) and, times shift / sqrt(D), to the
        # late keys: q . k * D^-1/2 gains `shift` for those keys (and noise of the usual size)
        u = np.where(_rng(c.seed, s0 + 8).random((c.Hkv, c.D)) < 0.5, -1.0, 1.0).astype(np.float32)
        q += np.repeat(u, c.Hq // c.Hkv, axis=0)[None, None, None]
        ku = u * np.float32(c.late_key_shift / math.sqrt(c.D))
        kb += ku[None, None, None]
        for b, plen in enumerate(c.prefix_lens):
            for t0 in range((c.late_from // bs) * bs, plen, bs):
                blk = tables[b, t0 // bs] if tables is not None else b * c.max_blocks + t0 // bs
                lo = max(c.late_from - t0, 0)
                kc[blk, :, lo:bs, :] += ku[:, None, :]

    k_scale = v_scale = None
    if c.kv_dtype == "fp8_e4m3":
        k_scale = (np.abs(kc).max(axis=(0, 2, 3)) / FP8_E4M3_MAX).astype(np.float32)
        v_scale = (np.abs(vc).max(axis=(0, 2, 3)) / FP8_E4M3_MAX).astype(np.float32)
        kc = kc / k_scale[None, :, None, None]
        vc = vc / v_scale[None, :, None, None]
    if c.branch_kv_dtype == "fp8_e4m3":
        if k_scale is None:
            raise ValueError("fp8 branch K/V needs an fp8 cache (shared scales)")
        kb = kb / k_scale[None, None, None, :, None]
        vb = vb / v_scale[None, None, None, :, None]

    return {
        "q": encode(q, c.q_dtype),
        "k_cache": encode(kc, c.kv_dtype),
        "v_cache": encode(vc, c.kv_dtype),
        "block_tables": tables,
        "prefix_lens": np.asarray(c.prefix_lens, dtype=np.int32),
        "k_branch": encode(kb, c.branch_kv_dtype),
        "v_branch": encode(vb, c.branch_kv_dtype),
        "k_scale": k_scale,
        "v_scale": v_scale,
    }


def _decode_for_sampling(bits: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return bits.astype(np.float64)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def make_accept_inputs(case: AcceptCase) -> Dict[str, np.ndarray]:
    """Target/draft logits, drafted tokens and the uniforms of one accept call (``draft_logits`` is None for a
    point-mass case).

    target ~ N(0, target_std^2); draft = target + N(0, noise^2) (or an
    independent N(0, target_std^2) when ``draft_noise_std`` is None).  The K
    drafted tokens are draws from the draft row's categorical distribution at
    the case's temperature, taken with the Gumbel-argmax construction on the
    *stored* (rounded) draft logits.  Uniforms are fp32 in [0, 1).
    """
    c = case
    t = _rng(c.seed, 100).standard_normal((c.NB, c.K + 1, c.V), dtype=np.float32) * np.float32(c.target_std)
    u_acc = _rng(c.seed, 103).random((c.NB, c.K), dtype=np.float32)
    u_smp = _rng(c.seed, 104).random((c.NB,), dtype=np.float32)
    if c.point_mass:
        # drafted tokens come without a distribution; the target row is peaked at them, as a language model's is at
        # a token that a lookup in the context proposes
        tokens = _rng(c.seed, 102).integers(0, c.V, size=(c.NB, c.K)).astype(np.int32)
        for nb in range(c.NB):
            for i in range(c.K):
                t[nb, i, tokens[nb, i]] += np.float32(c.peak)
        return {"target_logits": encode(t, c.logits_dtype), "draft_logits": None, "draft_tokens": tokens,
                "u_accept": u_acc, "u_sample": u_smp}
    if c.draft_noise_std is None:
        d = _rng(c.seed, 101).standard_normal((c.NB, c.K, c.V), dtype=np.float32) * np.float32(c.target_std)
    else:
        d = t[:, :c.K, :] + _rng(c.seed, 101).standard_normal((c.NB, c.K, c.V), dtype=np.float32) * np.float32(
            c.draft_noise_std)
    t_bits = encode(t, c.logits_dtype)
    d_bits = encode(d, c.logits_dtype)
    g = _rng(c.seed, 102)
    tokens = np.empty((c.NB, c.K), dtype=np.int32)
    for nb in range(c.NB):
        row = _decode_for_sampling(d_bits[nb], c.logits_dtype) / c.temperature
        gumbel = -np.log(-np.log(g.random(row.shape)))
        tokens[nb] = np.argmax(row + gumbel, axis=-1)
    return {"target_logits": t_bits, "draft_logits": d_bits, "draft_tokens": tokens, "u_accept": u_acc,
            "u_sample": u_smp}


def make_chain_inputs(case: AttnCase, chain_len: int, inp: Dict[str, Optional[np.ndarray]],
                      chain_vis: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """The drafted chain of the nested form: ``chain_len`` tokens of K/V ~ N(0,1) per request, ``[B, C, Hkv, D]`` in
    the branch storage type (fp8: the cache's scales, taken from ``inp``), and ``chain_vis [B, gamma]``, how many of
    them each branch sees.  Default: branch g sees the first ``g`` of ``gamma`` equal steps (the first branch none),
    the shape of a chain of drafted steps in which branch j is conditioned on steps 0..j-1."""
    c = case
    s0 = 16 * c.layer
    kch = _rng(c.seed, s0 + 8).standard_normal((c.B, chain_len, c.Hkv, c.D), dtype=np.float32)
    vch = _rng(c.seed, s0 + 9).standard_normal((c.B, chain_len, c.Hkv, c.D), dtype=np.float32)
    if c.branch_kv_dtype == "fp8_e4m3":
        kch = kch / inp["k_scale"][None, None, :, None]
        vch = vch / inp["v_scale"][None, None, :, None]
    if chain_vis is None:
        chain_vis = np.tile((np.arange(c.gamma) * chain_len) // c.gamma, (c.B, 1))
    return {"k_chain": encode(kch, c.branch_kv_dtype), "v_chain": encode(vch, c.branch_kv_dtype),
            "chain_vis": np.asarray(chain_vis, dtype=np.int32)}


def make_tree_inputs(case: AttnCase, width: int, depth: int, step_len: int,
                     inp: Dict[str, Optional[np.ndarray]]) -> Dict[str, np.ndarray]:
    """A draft tree (Section 3.1, multi-branch drafting): ``width`` alternative steps per position, ``depth``
    positions, every step ``step_len`` tokens of K/V ~ N(0,1).  The nodes are stored level by level (node ids 0..:
    the ``width`` children of node n follow each other), one segment per node, ``[B, nodes*step_len, Hkv, D]`` in
    the branch storage type.  Branch g is given the root path of node ``(3 g + b) mod (nodes + 1)`` (the extra
    value = no node: it sees only the prefix), i.e. ``seg_mask`` has the bits of that node and all its ancestors.
    Needs at most 64 nodes."""
    c = case
    nodes, level, parent = 0, [None], {}
    for _ in range(depth):
        nxt = []
        for par in level:
            for _ in range(width):
                parent[nodes] = par
                nxt.append(nodes)
                nodes += 1
        level = nxt
    if nodes > 64:
        raise ValueError("at most 64 nodes")
    C = nodes * step_len
    s0 = 16 * c.layer
    kp = _rng(c.seed, s0 + 11).standard_normal((c.B, C, c.Hkv, c.D), dtype=np.float32)
    vp = _rng(c.seed, s0 + 12).standard_normal((c.B, C, c.Hkv, c.D), dtype=np.float32)
    if c.branch_kv_dtype == "fp8_e4m3":
        kp = kp / inp["k_scale"][None, None, :, None]
        vp = vp / inp["v_scale"][None, None, :, None]
    seg = np.tile(np.repeat(np.arange(nodes, dtype=np.int32), step_len), (c.B, 1))
    mask = np.zeros((c.B, c.gamma), dtype=np.uint64)
    for b in range(c.B):
        for g in range(c.gamma):
            node = (3 * g + b) % (nodes + 1)
            node = None if node == nodes else node
            m = 0
            while node is not None:
                m |= 1 << node
                node = parent[node]
            mask[b, g] = m
    return {"k_pool": encode(kp, c.branch_kv_dtype), "v_pool": encode(vp, c.branch_kv_dtype), "pool_seg": seg,
            "seg_mask": mask}


def tree_parents(width: int, depth: int) -> np.ndarray:
    """Parent of every node of :func:`make_tree_inputs`'s tree (same numbering), -1 for the nodes of position 0."""
    par, level = [], [-1]
    for _ in range(depth):
        nxt = []
        for p in level:
            for _ in range(width):
                nxt.append(len(par))
                par.append(p)
        level = nxt
    return np.array(par, dtype=np.int32)


def make_commit_inputs(case: AttnCase, chain_len: int, decisions=None) -> Dict[str, np.ndarray]:
    """What a verification pass decided per request, for the KV commit: which branch survives (``src_branch``), how
    many tokens of the drafted chain (``n_chain``, 0..chain_len) and then of that branch (``n_own``, 0..L) are
    appended to the prefix.  Random unless ``decisions = (src_branch, n_chain, n_own)`` is given."""
    c = case
    if decisions is None:
        r = _rng(c.seed, 16 * c.layer + 10)
        decisions = (r.integers(0, c.gamma, size=c.B), r.integers(0, chain_len + 1, size=c.B),
                     r.integers(0, c.L + 1, size=c.B))
    src, nch, nown = (np.asarray(x, dtype=np.int32) for x in decisions)
    return {"src_branch": src, "n_chain": nch, "n_own": nown}


def with_layer(case: AttnCase, layer: int) -> AttnCase:
    return replace(case, layer=layer)


# ----------------------------------------------------------------------------- on-device generators

def make_attention_inputs_device(case: AttnCase, device="cuda"):
    """Same recipe as :func:`make_attention_inputs`, drawn on the GPU with torch's seeded generator.

    Used where the full-size tensors are too many to draw on the host in reasonable time (the 64-layer sweep:
    4.3 GB of fp8 cache).  The values differ from the numpy stream for the same seed; a checker reads the tensors
    back (``device_inputs_to_numpy``) so both sides still see identical bytes.
    """
    import torch

    c = case
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "fp8_e4m3": torch.float8_e4m3fn}
    gen = torch.Generator(device=device)
    gen.manual_seed((c.seed << 20) + 16 * c.layer + 1)
    B, bs = c.B, c.block_size
    blocks_needed = [-(-(p + c.spare_tokens) // bs) for p in c.prefix_lens]
    if c.paged:
        num_blocks = max(1, sum(blocks_needed))
        perm = torch.randperm(num_blocks, generator=gen, device=device).to(torch.int32)
        tables = torch.zeros((B, c.max_blocks), dtype=torch.int32, device=device)
        at = 0
        for b, nb in enumerate(blocks_needed):
            tables[b, :nb] = perm[at:at + nb]
            at += nb
    else:
        num_blocks = B * c.max_blocks
        tables = None

    def normal(shape):
        return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)

    q = normal((B, c.gamma, c.L, c.Hq, c.D))
    kb = normal((B, c.gamma, c.L, c.Hkv, c.D))
    vb = normal((B, c.gamma, c.L, c.Hkv, c.D))
    kc = normal((num_blocks, c.Hkv, bs, c.D))
    vc = normal((num_blocks, c.Hkv, bs, c.D))
    k_scale = v_scale = None
    if c.kv_dtype == "fp8_e4m3":
        k_scale = (kc.abs().amax(dim=(0, 2, 3)) / FP8_E4M3_MAX).float()
        v_scale = (vc.abs().amax(dim=(0, 2, 3)) / FP8_E4M3_MAX).float()
        kc = kc / k_scale[None, :, None, None]
        vc = vc / v_scale[None, :, None, None]
    if c.branch_kv_dtype == "fp8_e4m3":
        if k_scale is None:
            raise ValueError("fp8 branch K/V needs an fp8 cache (shared scales)")
        kb = (kb / k_scale[None, None, None, :, None]).clamp_(-FP8_E4M3_MAX, FP8_E4M3_MAX)
        vb = (vb / v_scale[None, None, None, :, None]).clamp_(-FP8_E4M3_MAX, FP8_E4M3_MAX)
    return {
        "q": q.to(tdt[c.q_dtype]),
        "k_cache": kc.to(tdt[c.kv_dtype]),
        "v_cache": vc.to(tdt[c.kv_dtype]),
        "block_tables": tables,
        "prefix_lens": torch.tensor(c.prefix_lens, dtype=torch.int32, device=device),
        "k_branch": kb.to(tdt[c.branch_kv_dtype]),
        "v_branch": vb.to(tdt[c.branch_kv_dtype]),
        "k_scale": k_scale,
        "v_scale": v_scale,
    }


def device_bits(t, dtype: str) -> Optional[np.ndarray]:
    """A device tensor as the storage array the host-side functions use (bit patterns for bf16/fp8)."""
    import torch

    if t is None:
        return None
    t = t.detach().cpu().contiguous()
    if dtype == "f32":
        return t.numpy()
    if dtype == "bf16":
        return t.view(torch.int16).numpy().view(np.uint16)
    if dtype == "fp8_e4m3":
        return t.view(torch.uint8).numpy()
    raise ValueError(dtype)


def device_inputs_to_numpy(case: AttnCase, dev: dict) -> Dict[str, Optional[np.ndarray]]:
    """Read the device tensors of one attention problem back as host storage arrays."""
    bits = device_bits
    return {
        "q": bits(dev["q"], case.q_dtype),
        "k_cache": bits(dev["k_cache"], case.kv_dtype),
        "v_cache": bits(dev["v_cache"], case.kv_dtype),
        "block_tables": None if dev["block_tables"] is None else dev["block_tables"].cpu().numpy(),
        "prefix_lens": dev["prefix_lens"].cpu().numpy(),
        "k_branch": bits(dev["k_branch"], case.branch_kv_dtype),
        "v_branch": bits(dev["v_branch"], case.branch_kv_dtype),
        "k_scale": None if dev["k_scale"] is None else dev["k_scale"].cpu().numpy(),
        "v_scale": None if dev["v_scale"] is None else dev["v_scale"].cpu().numpy(),
    }
