/*
 * la_verify.h -- C ABI of the MI355X (gfx950) verification hot path of
 * Lookahead Reasoning (arXiv 2506.19830).
 *
 * One verification pass of the target model expands the drafted reasoning
 * steps together (Section 3.1, Algorithm 1 "in parallel do": every candidate
 * continuation shares the prefix x_{1:t} and differs only in what was appended
 * after it), and token-level speculative decoding runs inside each step
 * (Section 2 "Speculative Decoding", Section 3.3).  The two entry points are
 * the two data-parallel pieces of that pass:
 *
 *   la_verify_attention  attention of gamma branches x L tokens against one
 *                        shared prefix KV cache plus branch-private KV
 *   la_spec_accept       accept length and one extra token per branch from
 *                        target/draft logits, drafted tokens and uniforms
 *
 * Conventions for every call
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary
 *     host memory.  All tensors are dense, row-major, 16-byte aligned.
 *   - The caller owns every buffer.  The library allocates no device memory,
 *     creates no stream and never synchronises; all work is enqueued on
 *     `hip_stream` (a hipStream_t passed as void*, NULL = the null stream).
 *   - Arguments are validated on the host before anything is launched; a
 *     rejected call launches nothing and returns a status code.  No exception
 *     or abort crosses this boundary.
 *   - Results are deterministic: the same inputs give bit-identical outputs.
 *   - Indices handed in by the caller (block ids, drafted token ids) are not
 *     range-checked on the device; out-of-range values are undefined behaviour.
 *   - Where an argument exists as a device array and as a host copy
 *     (prefix_lens / prefix_lens_host, chain_vis / chain_vis_host, pool_seg /
 *     pool_seg_host) the host copy is what is validated and what the launch
 *     and the workspace are sized from, and the kernels read the device array
 *     without checking it again: the two must hold the same values when the
 *     work runs, anything else is undefined behaviour.  (la_kv_commit's
 *     decisions are device-only and therefore clamped by the kernel.)
 *   - The library keeps no state between calls (what it caches -- the
 *     compute-unit count, per-kernel launch attributes, the address of
 *     la_spec_accept_static's scratch array -- is written once, under a lock,
 *     and only read afterwards), so calls may come from several host threads.
 *   - Benchmark aids (per-kernel event timing, calibration kernels, a self-test
 *     hook) are not part of this library: they are declared in
 *     la_verify_bench.h and exist only in libla_verify_bench.so, the same
 *     objects linked together with them.
 */
#ifndef LA_VERIFY_H
#define LA_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* only the la_* entry points below are exported from the shared library */
#define LA_API __attribute__((visibility("default")))

typedef enum {
  LA_OK = 0,
  LA_ERR_INVALID_ARG = 1,        /* NULL / negative / inconsistent argument            */
  LA_ERR_UNSUPPORTED = 2,        /* valid, but no kernel for this shape / dtype mix    */
  LA_ERR_WORKSPACE_TOO_SMALL = 3,
  LA_ERR_LAUNCH = 4              /* the HIP runtime refused a launch                   */
} la_status;

typedef enum {
  LA_F32 = 0,
  LA_BF16 = 1,
  LA_FP8_E4M3 = 2                /* OCP e4m3fn: no infinities, max 448                 */
} la_dtype;

/* ------------------------------------------------------------------------- *
 *  la_verify_attention
 *
 *  For request b, branch g, token i, query head h (KV head h / (Hq/Hkv)):
 *      keys/values = prefix tokens 0..P_b-1 of request b, then tokens 0..i of
 *                    branch g itself (causal inside the branch; other branches
 *                    are invisible -- Algorithm 1, prefixes x'_j)
 *      out = softmax(softmax_scale * q . K^T) V         lse = log sum exp
 *  The prefix cache is read once per KV head and shared by every branch and
 *  every query head of the group.
 *
 *  Supported combinations (anything else: LA_ERR_UNSUPPORTED)
 *      q f32,  cache f32,  branch f32,  out f32           head_dim 64 / 128 / 256
 *      q bf16, cache bf16, branch bf16, out bf16|f32      head_dim 64 / 128 / 256
 *      q bf16, cache fp8,  branch fp8|bf16, out bf16|f32  head_dim 64 / 128 / 256
 *  The bf16 / fp8 combinations run on the MFMA kernels at head_dim 128 and,
 *  like fp32 tensors, on the general kernel (fp32 arithmetic on exactly widened
 *  inputs, one wavefront per query row, no workspace) at head_dim 64 and 256;
 *  kernel_shape must be 0 there.
 *  fp8 storage is multiplied by k_scale[kv_head] / v_scale[kv_head]; a branch
 *  K/V stored as fp8 uses the same scales as the cache.  The scales are device
 *  arrays the host cannot inspect: they must be positive and finite (a zero,
 *  negative or non-finite scale gives undefined results, not an error code).
 *  Every query row must see at least one key (always true: a token sees
 *  itself), and K, V, Q must be finite.
 * ------------------------------------------------------------------------- */
typedef struct {
  int32_t num_requests;            /* B >= 1                                           */
  int32_t num_q_heads;             /* Hq, multiple of num_kv_heads                     */
  int32_t num_kv_heads;            /* Hkv                                              */
  int32_t head_dim;                /* D                                                */
  int32_t gamma;                   /* branches per request                             */
  int32_t branch_len;              /* L: tokens per branch (each a query and one private K,V) */
  int32_t block_size;              /* tokens per cache block: power of two >= 16       */
  int32_t max_blocks_per_request;  /* row stride of block_tables                       */
  int32_t q_dtype, kv_dtype, branch_kv_dtype, out_dtype;   /* la_dtype                 */
  float softmax_scale;             /* e.g. 1/sqrt(D); > 0                              */
  int32_t kv_split_tokens;         /* 0 = let the library choose how the prefix is cut
                                      into independently reduced chunks; otherwise the
                                      chunk length in tokens (multiple of 64)           */
  int32_t kernel_shape;            /* 0 = let the library choose the kernel shape of the
                                      bf16/fp8 path; k > 0 forces shape k (testing and
                                      tuning; numbering as la_attn_plan.kernel_shape
                                      reports it; LA_ERR_UNSUPPORTED when that shape
                                      cannot run the problem, LA_ERR_INVALID_ARG when
                                      there is no such shape)                           */
} la_attn_desc;

/* Bytes of device workspace la_verify_attention needs for this descriptor and
 * these prefix lengths (host array [B]).  0 is a valid answer. */
LA_API la_status la_verify_attention_workspace(const la_attn_desc *desc, const int32_t *prefix_lens_host,
                                        size_t *bytes_out);

/* What the library would launch for this descriptor and these prefix lengths
 * (host array [B]); chain_len > 0 asks for the nested / tree form.  A pure
 * function of its arguments and of the device's compute-unit count; nothing
 * is launched.  The answer is what the compute calls use, so a caller can
 * log it or size a sweep with it. */
typedef struct {
  int32_t path;               /* 1 = fp32 kernel, 2 = bf16/fp8 MFMA kernels                      */
  int32_t kernel_shape;       /* MFMA path: 1 = 256-row tiles, 3 LDS stages; 2 = 128-row tiles,
                                 2 stages; 3.. = streaming shapes (32-row blocks x key slices;
                                 fp8 cache and branch K/V: 3 = 2 x 4, 4 = 4 x 2, 5 = 8 x 1;
                                 bf16 cache and branch K/V: 6 = 8 x 1, 7 = 4 x 2)                */
  int32_t rows_per_workgroup; /* query rows (of one KV head) a workgroup owns                    */
  int32_t row_tiles;          /* workgroups per (KV head, chunk)                                 */
  int32_t chunk_tokens;       /* prefix tokens per independently reduced chunk                   */
  int32_t chunks_total;       /* chunks summed over the requests                                 */
  int32_t workgroups;         /* of the attention kernel                                         */
} la_attn_plan;
LA_API la_status la_verify_attention_plan(const la_attn_desc *desc, const int32_t *prefix_lens_host,
                                          int32_t chain_len, la_attn_plan *out);

LA_API la_status la_verify_attention(
    const la_attn_desc *desc,
    const void *q,                   /* dev [B, gamma, L, Hq, D]            q_dtype              */
    const void *k_cache,             /* dev [num_blocks, Hkv, block_size, D] kv_dtype (may be NULL if every prefix is empty) */
    const void *v_cache,             /* dev, same shape as k_cache                               */
    const int32_t *block_tables,     /* dev [B, max_blocks_per_request] physical block of each
                                        logical block; NULL => request b owns blocks
                                        b*max_blocks .. (b+1)*max_blocks-1 in order             */
    const int32_t *prefix_lens,      /* dev [B] prefix length of each request, 0 allowed; the
                                        last block may be partly filled                         */
    const int32_t *prefix_lens_host, /* host [B], same values (used to size the launch)         */
    const void *k_branch,            /* dev [B, gamma, L, Hkv, D]           branch_kv_dtype      */
    const void *v_branch,            /* dev, same shape                                          */
    const float *k_scale,            /* dev [Hkv] or NULL (=1); only read for fp8 storage        */
    const float *v_scale,            /* dev [Hkv] or NULL (=1)                                   */
    void *out,                       /* dev [B, gamma, L, Hq, D]            out_dtype            */
    float *lse,                      /* dev [B, gamma, L, Hq] natural-log sum-exp, or NULL       */
    void *workspace, size_t workspace_bytes, /* dev scratch, contents undefined before and after */
    void *hip_stream);

/* Nested branches (Algorithm 1: candidate j is conditioned on
 * x'_j = x (+) s^_0 .. s^_{j-1}, the common prefix followed by the first j
 * drafted steps).  The drafted steps of a request form one chain of chain_len
 * tokens; branch g sees the first chain_vis[b][g] of them, after the prefix
 * and before its own tokens (all chain tokens precede the branch's own, so
 * there is no mask inside the visible part).  chain_len == 0 is
 * la_verify_attention.  Same workspace as la_verify_attention. */
LA_API la_status la_verify_attention_nested(
    const la_attn_desc *desc, const void *q, const void *k_cache, const void *v_cache,
    const int32_t *block_tables, const int32_t *prefix_lens, const int32_t *prefix_lens_host,
    const void *k_branch, const void *v_branch,
    const void *k_chain,             /* dev [B, chain_len, Hkv, D]  branch_kv_dtype (fp8: the cache's
                                        scales); NULL when chain_len == 0                          */
    const void *v_chain,             /* dev, same shape                                          */
    int32_t chain_len,               /* C >= 0                                                   */
    const int32_t *chain_vis,        /* dev [B, gamma], each in 0..C                             */
    const int32_t *chain_vis_host,   /* host [B, gamma], same values (validated)                 */
    const float *k_scale, const float *v_scale, void *out, float *lse,
    void *workspace, size_t workspace_bytes, void *hip_stream);

/* Draft trees (Section 3.1, "Multi-Branch Drafting": W alternative steps per
 * position, so the drafted steps of a request form a tree).  The drafted
 * tokens of all tree nodes lie in one pool of pool_len tokens per request;
 * pool token c belongs to segment (tree node) pool_seg[b][c] in 0..63, and
 * branch g sees exactly the pool tokens whose segment bit is set in
 * seg_mask[b][g] -- the steps on its path from the root -- after the prefix
 * and before its own tokens (no mask inside what it sees: all of it precedes
 * the branch's own tokens).  At most 64 segments per request.  pool_len == 0
 * is la_verify_attention.  Same workspace as la_verify_attention. */
LA_API la_status la_verify_attention_tree(
    const la_attn_desc *desc, const void *q, const void *k_cache, const void *v_cache,
    const int32_t *block_tables, const int32_t *prefix_lens, const int32_t *prefix_lens_host,
    const void *k_branch, const void *v_branch,
    const void *k_pool,              /* dev [B, pool_len, Hkv, D]  branch_kv_dtype (fp8: the cache's
                                        scales); NULL when pool_len == 0                            */
    const void *v_pool,              /* dev, same shape                                           */
    int32_t pool_len,
    const int32_t *pool_seg,         /* dev [B, pool_len], each in 0..63                          */
    const int32_t *pool_seg_host,    /* host [B, pool_len], same values (validated)               */
    const uint64_t *seg_mask,        /* dev [B, gamma]                                            */
    const float *k_scale, const float *v_scale, void *out, float *lse,
    void *workspace, size_t workspace_bytes, void *hip_stream);

/* ------------------------------------------------------------------------- *
 *  la_kv_commit
 *
 *  Algorithm 1, once j* is known: the output  s^_0 .. s^_{j*-1} (+) s_{j*}
 *  becomes part of x.  For the cache that means: per request, the first
 *  n_chain[b] tokens of the drafted chain and then the first n_own[b] tokens
 *  of branch src_branch[b] are appended behind the prefix, token t of that
 *  sequence at position prefix_lens[b] + t through the block table, and
 *  new_prefix_lens[b] = prefix_lens[b] + n_chain[b] + n_own[b].  Everything
 *  else of the pass's private K/V is simply not copied.
 *
 *  The three decisions are device arrays (they come out of the accept step),
 *  so nothing here waits for the host; the kernel clamps them to their ranges
 *  (branch 0..gamma-1, n_chain 0..chain_len, n_own 0..branch_len) and never
 *  writes past max_blocks_per_request * block_size.  Because the host cannot
 *  see them, the block table must already map room for the most that can be
 *  appended: prefix_lens_host[b] + chain_len + branch_len positions, else
 *  LA_ERR_INVALID_ARG.
 *
 *  Storage: kv_dtype == branch_kv_dtype copies bytes (an fp8 branch already
 *  carries the cache's scales).  A bf16 source with an fp8 cache is quantised:
 *  code = e4m3fn(x / scale[head]), the quotient in fp32, round to nearest even,
 *  saturating at +-448.  Other pairs: LA_ERR_UNSUPPORTED.  head_dim % 16 == 0.
 *
 *  All layers of a model take the same decisions; `layers` (may be NULL = one
 *  layer) lets one call commit them all: layer l's tensors start l * stride
 *  ELEMENTS after layer 0's (cache_stride for k_cache and v_cache,
 *  branch_stride for k_branch and v_branch, chain_stride for the chain,
 *  scale_stride for k_scale and v_scale, 0 = shared scales); each layer's
 *  tensors must start 16-byte aligned.  block_tables, prefix_lens and the
 *  decisions are shared by all layers.
 *
 *  new_prefix_lens must not alias prefix_lens.  No workspace, no
 *  synchronisation, deterministic.  desc: the fields of the verification call
 *  (q_dtype, out_dtype, softmax_scale and kv_split_tokens are not used but
 *  must be valid).
 * ------------------------------------------------------------------------- */
typedef struct {
  int32_t num_layers;     /* 1..65535 */
  int64_t cache_stride;   /* elements */
  int64_t branch_stride;
  int64_t chain_stride;
  int64_t scale_stride;
} la_layer_strides;

LA_API la_status la_kv_commit(
    const la_attn_desc *desc,
    void *k_cache,                   /* dev, written: [num_blocks, Hkv, block_size, D] per layer   */
    void *v_cache,
    const int32_t *block_tables,     /* dev [B, max_blocks_per_request] or NULL (identity)          */
    const int32_t *prefix_lens,      /* dev [B]                                                     */
    const int32_t *prefix_lens_host, /* host [B], same values (room check)                         */
    const void *k_branch,            /* dev [B, gamma, L, Hkv, D] per layer                        */
    const void *v_branch,
    const void *k_chain,             /* dev [B, chain_len, Hkv, D] per layer; NULL if chain_len 0  */
    const void *v_chain,
    int32_t chain_len,
    const int32_t *src_branch,       /* dev [B]                                                     */
    const int32_t *n_chain,          /* dev [B]                                                     */
    const int32_t *n_own,            /* dev [B]                                                     */
    const float *k_scale,            /* dev [Hkv] per layer, or NULL = 1 (used when quantising)    */
    const float *v_scale,
    int32_t *new_prefix_lens,        /* dev [B], written                                           */
    const la_layer_strides *layers,  /* host, or NULL                                              */
    void *hip_stream);

/* la_kv_commit for a draft tree (Section 3.1, "Multi-Branch Drafting": of the
 * alternatives drafted for a position the accepted one is kept, the others
 * are discarded).  The drafted tokens lie in the pool of
 * la_verify_attention_tree; commit_mask[b] has the bits of the accepted nodes
 * (the path the verifier walked, see la_step_select_tree).  Per request the
 * pool tokens whose node is in commit_mask[b] are appended in pool order, then
 * the first n_own[b] tokens of branch src_branch[b];
 * new_prefix_lens[b] = prefix_lens[b] + (kept pool tokens) + n_own[b].
 * A pool_seg value outside 0..63 is never kept.  The block table must map
 * room for prefix_lens_host[b] + pool_len + branch_len positions.  Everything
 * else (storage pairs, layers, clamping, aliasing) is as in la_kv_commit;
 * chain_stride is the pool's layer stride. */
LA_API la_status la_kv_commit_tree(
    const la_attn_desc *desc, void *k_cache, void *v_cache, const int32_t *block_tables,
    const int32_t *prefix_lens, const int32_t *prefix_lens_host,
    const void *k_branch, const void *v_branch,
    const void *k_pool,              /* dev [B, pool_len, Hkv, D] per layer; NULL if pool_len 0    */
    const void *v_pool,
    int32_t pool_len,
    const int32_t *pool_seg,         /* dev [B, pool_len]; NULL if pool_len 0                      */
    const uint64_t *commit_mask,     /* dev [B]                                                     */
    const int32_t *src_branch,       /* dev [B]                                                     */
    const int32_t *n_own,            /* dev [B]                                                     */
    const float *k_scale, const float *v_scale,
    int32_t *new_prefix_lens,        /* dev [B], written                                           */
    const la_layer_strides *layers, void *hip_stream);

/* ------------------------------------------------------------------------- *
 *  la_spec_accept
 *
 *  Token-level speculative sampling (Section 2): with p_i = softmax(target
 *  row i / T) and q_i = softmax(draft row i / T), the drafted tokens x_0..
 *  x_{K-1} of a branch are examined in order; x_i is accepted when
 *  u_accept[i] * q_i(x_i) < p_i(x_i)  (probability min(1, p/q)); at the first
 *  rejection n the walk stops and next_token is drawn from
 *  norm(max(0, p_n - q_n)); when all K are accepted (n = K) next_token is
 *  drawn from the extra target row p_K.  Drawing is inverse-CDF in token
 *  order: the first v whose running sum exceeds u_sample * total.
 *
 *  draft_logits == NULL: the drafter proposed tokens without a distribution
 *  (the prompt-lookup / n-gram drafts of Section 4, Setup), i.e. q_i is the
 *  point mass at x_i: x_i is accepted when u_accept[i] < p_i(x_i), and after
 *  a rejection next_token is drawn from p_n with x_n removed.
 *
 *  top_k / top_p warp the target distributions p_i only (Section 4, Setup:
 *  temperature 0.6, top_p 0.95, top_k 20), in the order temperature, top-k,
 *  top-p; the draft distribution is used as given.
 *
 *  The accept test runs in fp32; the resampling row and the top-p masses are
 *  evaluated in fp64.
 *
 *  Logits may be -inf (a masked / constrained vocabulary): such a token has
 *  probability exactly 0, is never drawn, and is rejected when drafted
 *  (p = 0; also p = q = 0).  Every row must keep at least one finite logit;
 *  +inf and NaN logits give undefined results.
 * ------------------------------------------------------------------------- */
typedef struct {
  int32_t num_branches;   /* NB >= 1                                   */
  int32_t num_draft;      /* K  >= 1 drafted tokens per branch          */
  int32_t vocab;          /* V  >= 1                                   */
  int32_t logits_dtype;   /* LA_F32 or LA_BF16                          */
  float temperature;      /* T > 0, divides every logit                 */
  int32_t top_k;          /* 0 = off; else the target keeps a token iff fewer than top_k tokens
                             of its row have a larger logit (ties with the k-th stay)            */
  float top_p;            /* in (0, 1]; 1 = off; else, of what top_k kept, a token stays iff the
                             mass of the kept tokens with a larger logit is below top_p times
                             the kept mass; the target is then renormalised over what stays     */
} la_accept_desc;

LA_API la_status la_spec_accept_workspace(const la_accept_desc *desc, size_t *bytes_out);

LA_API la_status la_spec_accept(
    const la_accept_desc *desc,
    const void *target_logits,   /* dev [NB, K+1, V]                                      */
    const void *draft_logits,    /* dev [NB, K,   V], or NULL: point-mass draft at draft_tokens */
    const int32_t *draft_tokens, /* dev [NB, K]  each in 0..V-1                           */
    const float *u_accept,       /* dev [NB, K]  uniforms in [0,1)                        */
    const float *u_sample,       /* dev [NB]     uniforms in [0,1)                        */
    int32_t *accepted_len,       /* dev [NB] out: n in 0..K                               */
    int32_t *next_token,         /* dev [NB] out: in 0..V-1                               */
    float *accept_ratio,         /* dev [NB, K] out or NULL: p_i(x_i)/q_i(x_i) as computed,
                                    every position (also those after the rejection)      */
    void *workspace, size_t workspace_bytes, void *hip_stream);

/* la_spec_accept for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and kernels as la_spec_accept,
 * minus the workspace: the kernels use a scratch array of
 * LA_SPEC_ACCEPT_STATIC_MAX_BYTES that is part of the library's device image
 * (every GPU the library runs on holds its own copy until the process ends).
 * The call allocates and frees nothing; its first call on a device looks the
 * array's address up (do that once outside any capture).  A descriptor whose
 * la_spec_accept_workspace size exceeds the maximum is rejected with
 * LA_ERR_WORKSPACE_TOO_SMALL before anything is launched (NB = 32, K = 8,
 * V = 152064 needs 10.3 MB).  All calls on one GPU share that GPU's array:
 * calls that overlap on one GPU (two streams, two threads) race; calls on one
 * stream are ordered and need nothing cleared in between.  Leave
 * la_profile_enable off for such callers (event timing creates events). */
#define LA_SPEC_ACCEPT_STATIC_MAX_BYTES (16u << 20)
LA_API la_status la_spec_accept_static(
    const la_accept_desc *desc, const void *target_logits, const void *draft_logits,
    const int32_t *draft_tokens, const float *u_accept, const float *u_sample,
    int32_t *accepted_len, int32_t *next_token, float *accept_ratio, void *hip_stream);

/* ------------------------------------------------------------------------- *
 *  Step-level controller and budget planner (host only: every pointer below
 *  is a host pointer, nothing touches the GPU).
 *
 *  la_step_select -- Algorithm 1, verification and output construction.
 *  A pass has num_branches branches per request: branch j < num_branches-1
 *  checks draft step j (verdicts[b][j] != 0: the verifier accepted it), the
 *  last branch is the target's step behind all drafts.  j* = the first
 *  rejected draft, or num_branches-1 when none was rejected.  The output
 *  "accepted drafts, then the target's step j*" is what branch j* saw of the
 *  drafted chain plus what it produced, so the arguments of la_kv_commit are
 *  src_branch = j*, n_chain = chain_vis[b][j*], n_own = own_len[b][j*]
 *  (own_len: tokens of the target's step held by each branch).  Any of
 *  src_branch / n_chain / n_own may be NULL; chain_vis / own_len may be NULL
 *  when the output they feed is.
 *
 *  la_step_select_tree -- the same walk over a draft tree (Section 3.1,
 *  "Multi-Branch Drafting").  The tree has num_nodes <= 64 drafted steps, the
 *  same shape for every request: parent[n] in -1..n-1 (-1: a child of the
 *  root, i.e. an alternative for position 0), parents before children.  The
 *  target generates one step per tree prefix: branch 0 continues the bare
 *  prefix, branch 1+n continues the path that ends in node n (num_nodes + 1
 *  branches).  verdicts[b][n] != 0: the verifier accepted drafted step n as
 *  equivalent to the target's step of branch 1+parent[n].  The walk starts at
 *  the root and moves to an accepted child while there is one (several
 *  accepted alternatives: the one with the smallest node number); depth = the
 *  number of accepted steps, commit_mask = their node bits, src_branch = the
 *  branch of the node where the walk ended, n_own = own_len[b][src_branch].
 *  These are the arguments of la_kv_commit_tree.  A chain (parent[n] = n-1)
 *  gives la_step_select's result.
 *
 *  la_speedup_* -- closed forms, alpha in (0,1) the acceptance rate, c in
 *  (0,1) the draft's cost relative to the target, k >= 1 the depth:
 *    step level, sync  (Section 3.2):  (1-a^k) / ((1-a)(1-c+ck))
 *    step level, async (Section 3.2, Appendix B):
 *        k >= ceil(1/c):  1 / (c + (1-c)(1-a))
 *        else          :  (1-a^k) / ((1-a) + c [a - a^(k+1) - k(1-a)a^k])
 *    token level (Section 3.3, g): the sync form with (alpha2, c2, k2).
 *
 *  la_plan_budget -- Section 3.3:  max f(k1) g(k2)  over integers k1, k2 >= 1
 *  with ParallelDim_f * k2 <= budget, ParallelDim_f = k1 (sync) or
 *  min(ceil(1/c1), k1) (async).  Exhaustive over the feasible pairs; among
 *  equal maxima the smallest k1, then the smallest k2.  k1 = 1 is pure
 *  token-level speculation, k2 = 1 pure lookahead reasoning.
 * ------------------------------------------------------------------------- */
typedef struct {
  double alpha1, c1;     /* step level  */
  double alpha2, c2;     /* token level */
  int32_t budget;        /* M >= 1      */
  int32_t asynchronous;  /* 0 = sync f, else async f */
} la_plan_desc;

LA_API la_status la_step_select(int32_t num_requests, int32_t num_branches,
                                const uint8_t *verdicts,   /* [B, num_branches-1] */
                                const int32_t *chain_vis,  /* [B, num_branches]   */
                                const int32_t *own_len,    /* [B, num_branches]   */
                                int32_t *j_star,           /* [B] out             */
                                int32_t *src_branch, int32_t *n_chain, int32_t *n_own /* [B] out, optional */);
LA_API la_status la_step_select_tree(int32_t num_requests, int32_t num_nodes,
                                     const int32_t *parent,    /* [num_nodes]          */
                                     const uint8_t *verdicts,  /* [B, num_nodes]       */
                                     const int32_t *own_len,   /* [B, num_nodes + 1]   */
                                     int32_t *depth,           /* [B] out              */
                                     uint64_t *commit_mask,    /* [B] out              */
                                     int32_t *src_branch, int32_t *n_own /* [B] out, optional */);
LA_API la_status la_speedup_step_sync(double alpha1, double c1, int32_t k1, double *speedup);
LA_API la_status la_speedup_step_async(double alpha1, double c1, int32_t k1, double *speedup);
LA_API la_status la_speedup_token(double alpha2, double c2, int32_t k2, double *speedup);
LA_API la_status la_plan_budget(const la_plan_desc *desc, int32_t *k1, int32_t *k2, double *speedup);

/* ------------------------------------------------------------------------- *
 *  Diagnostics
 * ------------------------------------------------------------------------- */
/* Text of a status code; any integer is accepted (unknown ones give "unknown status"). */
LA_API const char *la_status_string(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* LA_VERIFY_H */
