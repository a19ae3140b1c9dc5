/*
 * CPU oracle for the verification hot path of Lookahead Reasoning
 * (arXiv 2506.19830).  TEST INFRASTRUCTURE ONLY: this file is the slow, plain
 * definition that the HIP library is checked against.  It shares no code,
 * header, table or helper with the GPU path and must never be called from the
 * product path.
 *
 * Everything is computed in fp64 from the exact bytes the GPU receives
 * (fp32 / bf16 / fp8-e4m3fn storage is widened exactly).
 *
 *   lao_verify_attention  -- Section 3.1 / Algorithm 1 ("in parallel do",
 *       prefixes x'_j): every drafted branch sees the common prefix x_{1:t}
 *       followed only by its own continuation.  For each branch the key/value
 *       sequence is written out explicitly as  prefix ++ branch tokens  and a
 *       textbook max-subtracted softmax attention is evaluated per query row.
 *       Nothing is shared between branches, nothing is tiled or split.
 *       Nested form (Algorithm 1: x'_j = x (+) s^_0 .. s^_{j-1}): the drafted
 *       steps form one chain of C tokens; branch g additionally sees the
 *       first chain_vis[g] chain tokens, between the prefix and its own tokens.
 *       Tree form (Section 3.1, "Multi-Branch Drafting": W alternative steps
 *       per position, a tree of drafted steps): the drafted steps of a request
 *       form a pool of C tokens, token c belonging to step (segment)
 *       pool_seg[c] in 0..63; branch g sees exactly the pool tokens whose
 *       segment bit is set in seg_mask[g] (the steps on its path from the
 *       root), in pool order, between the prefix and its own tokens.
 *   lao_attention_row_weights -- the softmax weights of one row (test hook
 *       for the "rows sum to one" pin).
 *   lao_spec_accept -- Section 2 ("Speculative Decoding"): the drafted tokens
 *       are examined in order, each accepted with probability min(1, p/q);
 *       at the first rejection the walk stops and one token is drawn from
 *       norm(max(0, p - q)); when all K survive, a bonus token is drawn from
 *       the (K+1)-th target row ("gamma+1 positions", Section 1).  Sampling is
 *       a sequential inverse-CDF walk.
 *   lao_kv_commit -- Algorithm 1, the step after j* is known (the output
 *       s^_0 .. s^_{j*-1} (+) s_{j*} is appended to x): for each request the
 *       first n_chain drafted-chain tokens and then the first n_own tokens of
 *       one chosen branch are written behind the prefix in the paged cache,
 *       one token at a time, and the prefix length grows by n_chain + n_own.
 *       Same storage type: the bytes are copied.  bf16 source into an fp8
 *       cache: code = nearest e4m3fn value (ties to even, saturating at 448)
 *       of  x / scale[head]  with the quotient taken in fp32, the precision
 *       the cache's writer computes in (the paper fixes none).
 *
 * Readings fixed here because the paper leaves them open (each is also listed
 * in the repository's design notes):
 *   - accept test is  u * q(x) < p(x)  with u in [0,1)  (so q(x)=0<p(x)
 *     accepts, p(x)=q(x)=0 rejects);                         parity unpinned
 *   - residual mass S == 0 after a rejection falls back to r = p_n;
 *                                                             parity unpinned
 *   - inverse CDF returns the first v whose running sum is > u*S (strict), so
 *     zero-mass tokens are never returned (pinned: a sample must have mass).
 * The first two items only matter on measure-zero / rounding-only inputs.
 *   - top-k / top-p (Section 4, Setup: temperature 0.6, top_p 0.95, top_k 20):
 *     the target distribution p is warped before the rule is applied, in the
 *     usual order temperature -> top-k -> top-p.  Both filters are read as
 *     predicates on a token's value, so that equal logits are never split:
 *       top-k keeps v  iff  #{u : l_u > l_v} < k          (ties with the k-th stay)
 *       top-p keeps v  iff  mass{u kept by top-k : l_u > l_v} < top_p * Z_k
 *     (Z_k the mass kept by top-k), then p is renormalised over what is kept.
 *     The draft distribution q is used as given.
 *   - draft_logits == NULL: the drafter proposes tokens without a distribution
 *     (Section 4, Setup: prompt-lookup / n-gram drafts), i.e. q_i is the point
 *     mass at the drafted token x_i.  The same rule then reads: accept with
 *     probability p_i(x_i); on rejection draw from p_n with x_n removed.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { LAO_F32 = 0, LAO_BF16 = 1, LAO_FP8_E4M3 = 2, LAO_F64 = 3 };

/* ---- exact widening of the storage formats --------------------------------- */

static double widen_bf16(uint16_t bits) {
  /* bfloat16 is the upper half of an IEEE binary32 */
  uint32_t w = (uint32_t)bits << 16;
  float f;
  memcpy(&f, &w, sizeof f);
  return (double)f;
}

static double widen_fp8_e4m3fn(uint8_t bits) {
  /* OCP 8-bit float, 1 sign / 4 exponent (bias 7) / 3 mantissa bits, no
   * infinities, S.1111.111 is NaN, largest finite value 448. */
  int sign = bits >> 7;
  int e = (bits >> 3) & 0xF;
  int m = bits & 0x7;
  double mag;
  if (e == 0xF && m == 0x7) return NAN;
  if (e == 0)
    mag = ldexp((double)m / 8.0, -6); /* subnormal */
  else
    mag = ldexp(1.0 + (double)m / 8.0, e - 7);
  return sign ? -mag : mag;
}

static double load_elem(const void *base, int dtype, int64_t idx) {
  switch (dtype) {
  case LAO_F32:
    return (double)((const float *)base)[idx];
  case LAO_BF16:
    return widen_bf16(((const uint16_t *)base)[idx]);
  case LAO_FP8_E4M3:
    return widen_fp8_e4m3fn(((const uint8_t *)base)[idx]);
  case LAO_F64:
    return ((const double *)base)[idx];
  default:
    return NAN;
  }
}

/* Test hook: widen n elements of the given storage type. */
int lao_widen(const void *src, int dtype, int64_t n, double *dst) {
  if (!src || !dst || dtype < 0 || dtype > LAO_F64) return 1;
  for (int64_t i = 0; i < n; ++i) dst[i] = load_elem(src, dtype, i);
  return 0;
}

/* ---- attention ---------------------------------------------------------------
 *
 * Tensor layouts (all row-major, host memory):
 *   q, k_branch, v_branch : [B, gamma, L, H, D]   (H = Hq for q, Hkv for k/v)
 *   k_cache, v_cache      : [num_blocks, Hkv, block_size, D]
 *   block_tables          : [B, max_blocks] int32, NULL => request b owns the
 *                           physical blocks b*max_blocks .. (b+1)*max_blocks-1
 *   prefix_lens           : [B] int32
 *   k_scale, v_scale      : [Hkv] fp32 multipliers applied to fp8 storage
 *                           (cache and, when stored as fp8, the branch K/V);
 *                           NULL => 1
 * A query row is named by  row_id = ((b*gamma + g)*L + i)*Hq + h.
 */

typedef struct {
  int B, gamma, L, Hq, Hkv, D, block_size, max_blocks;
  int q_dtype, kv_dtype, br_dtype;
  double scale;
  const void *q, *k_cache, *v_cache, *k_branch, *v_branch;
  const int32_t *block_tables, *prefix_lens;
  const float *k_scale, *v_scale;
  /* nested branches: a chain of C drafted tokens per request, [B, C, Hkv, D] in the branch dtype; branch g of
   * request b sees chain tokens 0 .. chain_vis[b*gamma+g]-1.  C == 0: flat form. */
  int C;
  const void *k_chain, *v_chain;
  const int32_t *chain_vis;
  /* tree form (pool_seg != NULL): the C tokens are a pool, token c of request b belongs to segment
   * pool_seg[b*C + c] in 0..63, and branch g sees the tokens whose segment bit is set in seg_mask[b*gamma + g] */
  const int32_t *pool_seg;
  const uint64_t *seg_mask;
} attn_problem;

/* does branch g of request b see chain / pool token c? */
static int sees_token(const attn_problem *a, int b, int g, int c) {
  if (a->pool_seg) {
    const int seg = a->pool_seg[(int64_t)b * a->C + c];
    return (int)((a->seg_mask[(int64_t)b * a->gamma + g] >> seg) & 1u);
  }
  return c < a->chain_vis[(int64_t)b * a->gamma + g];
}

/* number of chain / pool tokens branch g of request b sees */
static int visible_chain(const attn_problem *a, int b, int g) {
  int n = 0;
  for (int c = 0; c < a->C; ++c) n += sees_token(a, b, g, c);
  return n;
}

/* Writes the key and value sequence seen by branch g of request b on kv head
 * hk:  the P prefix tokens in logical order, then the visible part of the
 * drafted chain, then the branch's own L tokens.  kcat, vcat: [(P+vis+L), D]. */
static void concat_branch_kv(const attn_problem *a, int b, int g, int hk, double *kcat, double *vcat) {
  const int D = a->D;
  const int P = a->prefix_lens[b];
  const double ks = (a->k_scale && a->kv_dtype == LAO_FP8_E4M3) ? (double)a->k_scale[hk] : 1.0;
  const double vs = (a->v_scale && a->kv_dtype == LAO_FP8_E4M3) ? (double)a->v_scale[hk] : 1.0;
  for (int j = 0; j < P; ++j) {
    int64_t logical_block = j / a->block_size;
    int64_t phys = a->block_tables ? (int64_t)a->block_tables[(int64_t)b * a->max_blocks + logical_block]
                                   : (int64_t)b * a->max_blocks + logical_block;
    int64_t base = ((phys * a->Hkv + hk) * a->block_size + (j % a->block_size)) * D;
    for (int d = 0; d < D; ++d) {
      kcat[(int64_t)j * D + d] = load_elem(a->k_cache, a->kv_dtype, base + d) * ks;
      vcat[(int64_t)j * D + d] = load_elem(a->v_cache, a->kv_dtype, base + d) * vs;
    }
  }
  const double bks = (a->k_scale && a->br_dtype == LAO_FP8_E4M3) ? (double)a->k_scale[hk] : 1.0;
  const double bvs = (a->v_scale && a->br_dtype == LAO_FP8_E4M3) ? (double)a->v_scale[hk] : 1.0;
  int vis = 0; /* visible tokens written so far; they keep their order */
  for (int c = 0; c < a->C; ++c) {
    if (!sees_token(a, b, g, c)) continue;
    int64_t base = (((int64_t)b * a->C + c) * a->Hkv + hk) * D;
    for (int d = 0; d < D; ++d) {
      kcat[(int64_t)(P + vis) * D + d] = load_elem(a->k_chain, a->br_dtype, base + d) * bks;
      vcat[(int64_t)(P + vis) * D + d] = load_elem(a->v_chain, a->br_dtype, base + d) * bvs;
    }
    ++vis;
  }
  for (int i = 0; i < a->L; ++i) {
    int64_t base = ((((int64_t)b * a->gamma + g) * a->L + i) * a->Hkv + hk) * D;
    for (int d = 0; d < D; ++d) {
      kcat[(int64_t)(P + vis + i) * D + d] = load_elem(a->k_branch, a->br_dtype, base + d) * bks;
      vcat[(int64_t)(P + vis + i) * D + d] = load_elem(a->v_branch, a->br_dtype, base + d) * bvs;
    }
  }
}

/* Softmax weights of query row (b,g,i,h) over its n = P+i+1 visible keys.
 * w: [n]; returns log-sum-exp of the scaled scores through *lse. */
static void row_softmax(const attn_problem *a, int b, int g, int i, int h, const double *kcat, int64_t n, double *w,
                        double *lse) {
  const int D = a->D;
  int64_t qbase = ((((int64_t)b * a->gamma + g) * a->L + i) * a->Hq + h) * D;
  double qrow[D];
  for (int d = 0; d < D; ++d) qrow[d] = load_elem(a->q, a->q_dtype, qbase + d);
  double m = -INFINITY;
  for (int64_t j = 0; j < n; ++j) {
    double s = 0.0;
    for (int d = 0; d < D; ++d) s += qrow[d] * kcat[j * D + d];
    s *= a->scale;
    w[j] = s;
    if (s > m) m = s;
  }
  double z = 0.0;
  for (int64_t j = 0; j < n; ++j) {
    w[j] = exp(w[j] - m);
    z += w[j];
  }
  for (int64_t j = 0; j < n; ++j) w[j] /= z;
  *lse = m + log(z);
}

static int check_problem(const attn_problem *a) {
  if (a->B < 1 || a->gamma < 1 || a->L < 1 || a->Hq < 1 || a->Hkv < 1 || a->D < 1 || a->D > 1024) return 1;
  if (a->Hq % a->Hkv) return 1;
  if (a->block_size < 1 || a->max_blocks < 0) return 1;
  if (!a->q || !a->k_branch || !a->v_branch || !a->prefix_lens) return 1;
  for (int b = 0; b < a->B; ++b) {
    if (a->prefix_lens[b] < 0) return 1;
    if ((int64_t)a->prefix_lens[b] > (int64_t)a->max_blocks * a->block_size) return 1;
    if (a->prefix_lens[b] > 0 && (!a->k_cache || !a->v_cache)) return 1;
  }
  if (a->C < 0) return 1;
  if (a->C > 0) {
    if (!a->k_chain || !a->v_chain) return 1;
    if (a->pool_seg) {
      if (!a->seg_mask) return 1;
      for (int64_t t = 0; t < (int64_t)a->B * a->C; ++t)
        if (a->pool_seg[t] < 0 || a->pool_seg[t] > 63) return 1;
    } else {
      if (!a->chain_vis) return 1;
      for (int64_t t = 0; t < (int64_t)a->B * a->gamma; ++t)
        if (a->chain_vis[t] < 0 || a->chain_vis[t] > a->C) return 1;
    }
  }
  return 0;
}

/* out: [n_rows, D] fp64, lse: [n_rows] fp64 or NULL.  row_ids == NULL means
 * every row in order (n_rows must then equal B*gamma*L*Hq). */
static int verify_attention(attn_problem a, const int64_t *row_ids, int64_t n_rows, double *out, double *lse) {
  const int B = a.B, gamma = a.gamma, L = a.L, Hq = a.Hq, Hkv = a.Hkv, D = a.D;
  const int32_t *prefix_lens = a.prefix_lens;
  if (check_problem(&a) || !out) return 1;
  const int64_t total = (int64_t)B * gamma * L * Hq;
  if (!row_ids && n_rows != total) return 1;
  for (int64_t r = 0; row_ids && r < n_rows; ++r)
    if (row_ids[r] < 0 || row_ids[r] >= total) return 1;
  const int G = Hq / Hkv;
  const int64_t groups = (int64_t)B * gamma * Hkv;
  int failed = 0;

#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t grp = 0; grp < groups; ++grp) {
    const int hk = (int)(grp % Hkv);
    const int g = (int)((grp / Hkv) % gamma);
    const int b = (int)(grp / ((int64_t)Hkv * gamma));
    /* does any requested row belong to this (request, branch, kv head)? */
    int wanted = (row_ids == NULL);
    for (int64_t r = 0; !wanted && r < n_rows; ++r) {
      int64_t id = row_ids[r];
      int h = (int)(id % Hq);
      int64_t t = id / Hq / L; /* = b*gamma + g */
      if (h / G == hk && t == (int64_t)b * gamma + g) wanted = 1;
    }
    if (!wanted) continue;
    const int P = prefix_lens[b];
    const int vis = visible_chain(&a, b, g);
    const int64_t n_max = (int64_t)P + vis + L;
    double *kcat = malloc(sizeof(double) * n_max * D);
    double *vcat = malloc(sizeof(double) * n_max * D);
    double *w = malloc(sizeof(double) * n_max);
    if (!kcat || !vcat || !w) {
      failed = 1;
      free(kcat), free(vcat), free(w);
      continue;
    }
    concat_branch_kv(&a, b, g, hk, kcat, vcat);
    const int64_t n_iter = row_ids ? n_rows : (int64_t)L * G;
    for (int64_t it = 0; it < n_iter; ++it) {
      int i, h;
      int64_t slot;
      if (row_ids) {
        int64_t id = row_ids[it];
        h = (int)(id % Hq);
        i = (int)((id / Hq) % L);
        if (h / G != hk || id / Hq / L != (int64_t)b * gamma + g) continue;
        slot = it;
      } else {
        i = (int)(it / G);
        h = hk * G + (int)(it % G);
        slot = ((((int64_t)b * gamma + g) * L + i) * Hq + h);
      }
      const int64_t n = (int64_t)P + vis + i + 1; /* causal inside the branch */
      double row_lse;
      row_softmax(&a, b, g, i, h, kcat, n, w, &row_lse);
      double *o = out + slot * D;
      for (int d = 0; d < D; ++d) o[d] = 0.0;
      for (int64_t j = 0; j < n; ++j)
        for (int d = 0; d < D; ++d) o[d] += w[j] * vcat[j * D + d];
      if (lse) lse[slot] = row_lse;
    }
    free(kcat), free(vcat), free(w);
  }
  return failed;
}

int lao_verify_attention_nested(int B, int gamma, int L, int Hq, int Hkv, int D, int block_size, int max_blocks,
                                int q_dtype, int kv_dtype, int br_dtype, double scale, const void *q,
                                const void *k_cache, const void *v_cache, const int32_t *block_tables,
                                const int32_t *prefix_lens, const void *k_branch, const void *v_branch,
                                const float *k_scale, const float *v_scale, int chain_len, const void *k_chain,
                                const void *v_chain, const int32_t *chain_vis, const int64_t *row_ids, int64_t n_rows,
                                double *out, double *lse) {
  attn_problem a = {B,  gamma,   L,       Hq,       Hkv,      D,           block_size, max_blocks, q_dtype, kv_dtype, br_dtype,
                    scale, q, k_cache, v_cache, k_branch, v_branch, block_tables, prefix_lens, k_scale, v_scale,
                    chain_len, k_chain, v_chain, chain_vis, NULL, NULL};
  return verify_attention(a, row_ids, n_rows, out, lse);
}

int lao_verify_attention_tree(int B, int gamma, int L, int Hq, int Hkv, int D, int block_size, int max_blocks,
                              int q_dtype, int kv_dtype, int br_dtype, double scale, const void *q,
                              const void *k_cache, const void *v_cache, const int32_t *block_tables,
                              const int32_t *prefix_lens, const void *k_branch, const void *v_branch,
                              const float *k_scale, const float *v_scale, int pool_len, const void *k_pool,
                              const void *v_pool, const int32_t *pool_seg, const uint64_t *seg_mask,
                              const int64_t *row_ids, int64_t n_rows, double *out, double *lse) {
  attn_problem a = {B,  gamma,   L,       Hq,       Hkv,      D,           block_size, max_blocks, q_dtype, kv_dtype, br_dtype,
                    scale, q, k_cache, v_cache, k_branch, v_branch, block_tables, prefix_lens, k_scale, v_scale,
                    pool_len, k_pool, v_pool, NULL, pool_seg, seg_mask};
  if (pool_len > 0 && !pool_seg) return 1;
  return verify_attention(a, row_ids, n_rows, out, lse);
}

int lao_verify_attention(int B, int gamma, int L, int Hq, int Hkv, int D, int block_size, int max_blocks, int q_dtype,
                         int kv_dtype, int br_dtype, double scale, const void *q, const void *k_cache,
                         const void *v_cache, const int32_t *block_tables, const int32_t *prefix_lens,
                         const void *k_branch, const void *v_branch, const float *k_scale, const float *v_scale,
                         const int64_t *row_ids, int64_t n_rows, double *out, double *lse) {
  return lao_verify_attention_nested(B, gamma, L, Hq, Hkv, D, block_size, max_blocks, q_dtype, kv_dtype, br_dtype,
                                     scale, q, k_cache, v_cache, block_tables, prefix_lens, k_branch, v_branch,
                                     k_scale, v_scale, 0, NULL, NULL, NULL, row_ids, n_rows, out, lse);
}

/* Softmax weights of one row over its P+i+1 visible keys (prefix first, then
 * branch tokens 0..i).  w must hold prefix_lens[b]+i+1 doubles. */
int lao_attention_row_weights(int B, int gamma, int L, int Hq, int Hkv, int D, int block_size, int max_blocks,
                              int q_dtype, int kv_dtype, int br_dtype, double scale, const void *q,
                              const void *k_cache, const void *v_cache, const int32_t *block_tables,
                              const int32_t *prefix_lens, const void *k_branch, const void *v_branch,
                              const float *k_scale, const float *v_scale, int64_t row_id, double *w) {
  attn_problem a = {B,  gamma,   L,       Hq,       Hkv,      D,           block_size, max_blocks, q_dtype, kv_dtype, br_dtype,
                    scale, q, k_cache, v_cache, k_branch, v_branch, block_tables, prefix_lens, k_scale, v_scale,
                    0, NULL, NULL, NULL, NULL, NULL};
  if (check_problem(&a) || !w) return 1;
  if (row_id < 0 || row_id >= (int64_t)B * gamma * L * Hq) return 1;
  const int h = (int)(row_id % Hq);
  const int i = (int)((row_id / Hq) % L);
  const int g = (int)((row_id / Hq / L) % gamma);
  const int b = (int)(row_id / Hq / L / gamma);
  const int hk = h / (Hq / Hkv);
  const int64_t n_max = (int64_t)prefix_lens[b] + L;
  double *kcat = malloc(sizeof(double) * n_max * D);
  double *vcat = malloc(sizeof(double) * n_max * D);
  if (!kcat || !vcat) {
    free(kcat), free(vcat);
    return 1;
  }
  concat_branch_kv(&a, b, g, hk, kcat, vcat);
  double lse;
  row_softmax(&a, b, g, i, h, kcat, (int64_t)prefix_lens[b] + i + 1, w, &lse);
  free(kcat), free(vcat);
  return 0;
}

/* ---- speculative accept / resample -------------------------------------------
 *
 *   target_logits [NB, K+1, V], draft_logits [NB, K, V]  (storage dtype given)
 *   draft_tokens  [NB, K] int32,  u_accept [NB, K] fp32,  u_sample [NB] fp32
 * outputs
 *   accepted_len [NB] (0..K), next_token [NB] (0..V-1)
 *   ratio   [NB, K]  p(x)/q(x) at every examined position, NaN elsewhere
 *   margin  [NB, K]  |u - min(1, p/q)| at every examined position, +inf elsewhere
 *   cdf_lo, cdf_hi [NB]  normalised CDF edges of the returned token
 *   (any of the four diagnostic outputs may be NULL)
 */

static void softmax_row(const void *logits, int dtype, int64_t base, int V, double temperature, double *p) {
  double m = -INFINITY;
  for (int v = 0; v < V; ++v) {
    p[v] = load_elem(logits, dtype, base + v) / temperature;
    if (p[v] > m) m = p[v];
  }
  double z = 0.0;
  for (int v = 0; v < V; ++v) {
    p[v] = exp(p[v] - m);
    z += p[v];
  }
  for (int v = 0; v < V; ++v) p[v] /= z;
}

typedef struct {
  double v;
  int id;
} ranked;

static int by_value_desc_then_id(const void *a, const void *b) {
  const ranked *x = a, *y = b;
  if (x->v > y->v) return -1;
  if (x->v < y->v) return 1;
  return (x->id > y->id) - (x->id < y->id);
}

/* Top-k then top-p on a normalised row p (see the header comment for the two predicates); p is renormalised over the
 * kept tokens.  *margin (if not NULL) receives the smallest |M - top_p*Z_k| / Z_k over the cumulative masses M that
 * were compared with the top-p threshold: a measure of how close the kept set is to changing. */
static int warp_row(double *p, int V, int top_k, double top_p, double *margin) {
  if (margin) *margin = INFINITY;
  const int use_k = top_k > 0 && top_k < V, use_p = top_p < 1.0;
  if (!use_k && !use_p) return 0;
  ranked *r = malloc(sizeof(ranked) * V);
  if (!r) return 1;
  for (int v = 0; v < V; ++v) r[v].v = p[v], r[v].id = v;
  qsort(r, V, sizeof(ranked), by_value_desc_then_id);
  int kept = V;
  if (use_k) {
    kept = top_k;
    while (kept < V && r[kept].v == r[top_k - 1].v) ++kept; /* ties with the k-th largest stay */
  }
  if (use_p) {
    double zk = 0.0;
    for (int j = 0; j < kept; ++j) zk += r[j].v;
    const double T = top_p * zk;
    double M = 0.0, mg = INFINITY;
    int j = 0;
    while (j < kept) {
      const double d = fabs(M - T) / zk;
      if (d < mg) mg = d;
      if (!(M < T)) break; /* the tokens of this value have mass >= T above them */
      int e = j;
      double gm = 0.0;
      while (e < kept && r[e].v == r[j].v) gm += r[e++].v;
      M += gm;
      j = e;
    }
    kept = j;
    if (margin) *margin = mg;
  }
  double z = 0.0;
  for (int j = 0; j < kept; ++j) z += r[j].v;
  for (int j = kept; j < V; ++j) p[r[j].id] = 0.0;
  for (int j = 0; j < kept; ++j) p[r[j].id] = r[j].v / z;
  free(r);
  return 0;
}

/* Test hook: the warped distribution of one logit row. */
int lao_warp_probs(const void *logits, int dtype, int V, double temperature, int top_k, double top_p, double *p_out,
                   double *margin) {
  if (!logits || !p_out || V < 1 || !(temperature > 0.0) || !(top_p > 0.0)) return 1;
  softmax_row(logits, dtype, 0, V, temperature, p_out);
  return warp_row(p_out, V, top_k, top_p, margin);
}

int lao_spec_accept_warped(int NB, int K, int V, int logits_dtype, double temperature, int top_k, double top_p,
                           const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
                           const float *u_accept, const float *u_sample, int32_t *accepted_len, int32_t *next_token,
                           double *ratio, double *margin, double *cdf_lo, double *cdf_hi, double *warp_margin) {
  if (NB < 1 || K < 1 || V < 1 || !(temperature > 0.0) || !(top_p > 0.0) || top_k < 0) return 1;
  if (!target_logits || !draft_tokens || !u_accept || !u_sample || !accepted_len || !next_token) return 1;
  for (int64_t t = 0; t < (int64_t)NB * K; ++t)
    if (draft_tokens[t] < 0 || draft_tokens[t] >= V) return 1;
  int failed = 0;

#pragma omp parallel for schedule(dynamic, 1)
  for (int nb = 0; nb < NB; ++nb) {
    double *p = malloc(sizeof(double) * V);
    double *q = malloc(sizeof(double) * V);
    double *r = malloc(sizeof(double) * V);
    if (!p || !q || !r) {
      failed = 1;
      free(p), free(q), free(r);
      continue;
    }
    for (int i = 0; i < K; ++i) {
      if (ratio) ratio[(int64_t)nb * K + i] = NAN;
      if (margin) margin[(int64_t)nb * K + i] = INFINITY;
    }
    double wm = INFINITY, wm_row; /* closest top-p decision over the target rows this branch evaluates */
    /* examine the drafted tokens in order; stop at the first rejection */
    int n = K;
    for (int i = 0; i < K; ++i) {
      softmax_row(target_logits, logits_dtype, ((int64_t)nb * (K + 1) + i) * V, V, temperature, p);
      if (warp_row(p, V, top_k, top_p, &wm_row)) failed = 1;
      if (wm_row < wm) wm = wm_row;
      const int x = draft_tokens[(int64_t)nb * K + i];
      if (draft_logits) {
        softmax_row(draft_logits, logits_dtype, ((int64_t)nb * K + i) * V, V, temperature, q);
      } else { /* point-mass draft */
        for (int v = 0; v < V; ++v) q[v] = 0.0;
        q[x] = 1.0;
      }
      const double u = (double)u_accept[(int64_t)nb * K + i];
      if (ratio) ratio[(int64_t)nb * K + i] = p[x] / q[x];
      if (margin) {
        double thr = (q[x] > 0.0) ? fmin(1.0, p[x] / q[x]) : (p[x] > 0.0 ? 1.0 : 0.0);
        margin[(int64_t)nb * K + i] = fabs(u - thr);
      }
      const int accept = (u * q[x] < p[x]);
      if (!accept) {
        n = i;
        break;
      }
    }
    /* distribution of the one extra token */
    double S = 0.0;
    if (n < K) {
      /* p and q still hold the rows of position n */
      for (int v = 0; v < V; ++v) {
        r[v] = p[v] - q[v];
        if (r[v] < 0.0) r[v] = 0.0;
        S += r[v];
      }
      if (!(S > 0.0)) {
        S = 0.0;
        for (int v = 0; v < V; ++v) {
          r[v] = p[v];
          S += r[v];
        }
      }
    } else {
      softmax_row(target_logits, logits_dtype, ((int64_t)nb * (K + 1) + K) * V, V, temperature, r);
      if (warp_row(r, V, top_k, top_p, &wm_row)) failed = 1;
      if (wm_row < wm) wm = wm_row;
      for (int v = 0; v < V; ++v) S += r[v];
    }
    /* inverse-CDF walk */
    const double thr = (double)u_sample[nb] * S;
    double c = 0.0, lo = 0.0;
    int tok = -1;
    for (int v = 0; v < V; ++v) {
      lo = c;
      c += r[v];
      if (c > thr) {
        tok = v;
        break;
      }
    }
    if (tok < 0) { /* only reachable through rounding: last token with mass */
      for (int v = V - 1; v >= 0; --v)
        if (r[v] > 0.0) {
          tok = v;
          break;
        }
      lo = c - r[tok];
    }
    accepted_len[nb] = n;
    next_token[nb] = tok;
    if (cdf_lo) cdf_lo[nb] = lo / S;
    if (cdf_hi) cdf_hi[nb] = (lo + r[tok]) / S;
    if (warp_margin) warp_margin[nb] = wm;
    free(p), free(q), free(r);
  }
  return failed;
}

int lao_spec_accept(int NB, int K, int V, int logits_dtype, double temperature, const void *target_logits,
                    const void *draft_logits, const int32_t *draft_tokens, const float *u_accept,
                    const float *u_sample, int32_t *accepted_len, int32_t *next_token, double *ratio, double *margin,
                    double *cdf_lo, double *cdf_hi) {
  return lao_spec_accept_warped(NB, K, V, logits_dtype, temperature, 0, 1.0, target_logits, draft_logits, draft_tokens,
                                u_accept, u_sample, accepted_len, next_token, ratio, margin, cdf_lo, cdf_hi, NULL);
}

/* ---- KV commit ------------------------------------------------------------------ */

/* Nearest e4m3fn code of y (finite): candidates are the 127 non-negative finite values, the nearest wins, a tie goes
 * to the code with an even mantissa, magnitudes beyond the largest finite value 448 saturate to it. */
static uint8_t nearest_fp8_e4m3fn(float y) {
  double a = fabs((double)y);
  int best = 0;
  double best_d = INFINITY;
  for (int code = 0; code < 127; ++code) {
    double d = fabs(widen_fp8_e4m3fn((uint8_t)code) - a);
    if (d < best_d || (d == best_d && (code & 1) == 0)) {
      best = code;
      best_d = d;
    }
  }
  if (a > 448.0) best = 126;
  return (uint8_t)(best | (signbit(y) ? 0x80 : 0));
}

static size_t storage_size(int dtype) {
  return dtype == LAO_F32 ? 4 : dtype == LAO_BF16 ? 2 : dtype == LAO_FP8_E4M3 ? 1 : 8;
}

/* One token row of one kv head: D elements from src (storage src_dtype) to dst (storage dst_dtype). */
static int commit_row(const void *src, int src_dtype, int64_t src_idx, void *dst, int dst_dtype, int64_t dst_idx,
                      int D, const float *scale, int hk) {
  if (src_dtype == dst_dtype) {
    size_t sz = storage_size(src_dtype);
    memcpy((char *)dst + (size_t)dst_idx * sz, (const char *)src + (size_t)src_idx * sz, (size_t)D * sz);
    return 0;
  }
  if (src_dtype == LAO_BF16 && dst_dtype == LAO_FP8_E4M3) {
    const float s = scale ? scale[hk] : 1.0f;
    for (int d = 0; d < D; ++d) {
      const float x = (float)widen_bf16(((const uint16_t *)src)[src_idx + d]);
      const float y = x / s; /* fp32 quotient, correctly rounded */
      ((uint8_t *)dst)[dst_idx + d] = nearest_fp8_e4m3fn(y);
    }
    return 0;
  }
  return 1;
}

/* k_cache / v_cache are updated in place.  src_branch [B] in 0..gamma-1, n_chain [B] in 0..C, n_own [B] in 0..L.
 * new_prefix_lens [B] receives prefix_lens + n_chain + n_own.  The block table must already map every position
 * that is written. */
/* One request's appended sequence, shared by the chain and the tree form: `n_drafted` drafted tokens (their row
 * numbers inside the request's chain / pool are drafted[0..n_drafted)), then own tokens 0..n_own-1 of src_branch. */
static int commit_request(int b, int gamma, int L, int Hkv, int D, int block_size, int max_blocks, int kv_dtype,
                          int br_dtype, void *k_cache, void *v_cache, const int32_t *block_tables, int pos,
                          const void *k_branch, const void *v_branch, int C, const void *k_drafted,
                          const void *v_drafted, const int *drafted, int n_drafted, int src_branch, int n_own,
                          const float *k_scale, const float *v_scale) {
  for (int t = 0; t < n_drafted + n_own; ++t, ++pos) {
    const int from_drafted = t < n_drafted;
    const int64_t logical_block = pos / block_size;
    const int64_t phys = block_tables ? (int64_t)block_tables[(int64_t)b * max_blocks + logical_block]
                                      : (int64_t)b * max_blocks + logical_block;
    for (int hk = 0; hk < Hkv; ++hk) {
      const int64_t dst = ((phys * Hkv + hk) * block_size + (pos % block_size)) * D;
      int64_t src;
      const void *ks, *vs;
      if (from_drafted) {
        src = (((int64_t)b * C + drafted[t]) * Hkv + hk) * D;
        ks = k_drafted, vs = v_drafted;
      } else {
        const int i = t - n_drafted;
        src = ((((int64_t)b * gamma + src_branch) * L + i) * Hkv + hk) * D;
        ks = k_branch, vs = v_branch;
      }
      if (commit_row(ks, br_dtype, src, k_cache, kv_dtype, dst, D, k_scale, hk)) return 2;
      if (commit_row(vs, br_dtype, src, v_cache, kv_dtype, dst, D, v_scale, hk)) return 2;
    }
  }
  return 0;
}

int lao_kv_commit(int B, int gamma, int L, int Hkv, int D, int block_size, int max_blocks, int kv_dtype, int br_dtype,
                  void *k_cache, void *v_cache, const int32_t *block_tables, const int32_t *prefix_lens,
                  const void *k_branch, const void *v_branch, int C, const void *k_chain, const void *v_chain,
                  const int32_t *src_branch, const int32_t *n_chain, const int32_t *n_own, const float *k_scale,
                  const float *v_scale, int32_t *new_prefix_lens) {
  if (B < 1 || gamma < 1 || L < 1 || Hkv < 1 || D < 1 || block_size < 1 || C < 0) return 1;
  if (!k_cache || !v_cache || !prefix_lens || !k_branch || !v_branch || !src_branch || !n_chain || !n_own ||
      !new_prefix_lens)
    return 1;
  if (C > 0 && (!k_chain || !v_chain)) return 1;
  for (int b = 0; b < B; ++b) {
    if (src_branch[b] < 0 || src_branch[b] >= gamma || n_chain[b] < 0 || n_chain[b] > C || n_own[b] < 0 ||
        n_own[b] > L)
      return 1;
    if ((int64_t)prefix_lens[b] + n_chain[b] + n_own[b] > (int64_t)max_blocks * block_size) return 1;
  }
  int *rows = (int *)malloc(sizeof(int) * (size_t)(C > 0 ? C : 1));
  if (!rows) return 3;
  for (int c = 0; c < C; ++c) rows[c] = c; /* the accepted part of a chain is its first n_chain tokens */
  int rc = 0;
  for (int b = 0; b < B && !rc; ++b) {
    rc = commit_request(b, gamma, L, Hkv, D, block_size, max_blocks, kv_dtype, br_dtype, k_cache, v_cache,
                        block_tables, prefix_lens[b], k_branch, v_branch, C, k_chain, v_chain, rows, n_chain[b],
                        src_branch[b], n_own[b], k_scale, v_scale);
    new_prefix_lens[b] = prefix_lens[b] + n_chain[b] + n_own[b];
  }
  free(rows);
  return rc;
}

/* Tree form (Section 3.1, "Multi-Branch Drafting": of the alternatives drafted for a position the accepted one is
 * kept, the others are discarded).  The drafted tokens of all tree nodes lie in one pool [B, C, Hkv, D]; pool token c
 * belongs to node pool_seg[b][c] in 0..63.  commit_mask[b] has the bits of the accepted nodes (the path the verifier
 * walked); their tokens are appended in pool order, then own tokens 0..n_own-1 of src_branch. */
int lao_kv_commit_tree(int B, int gamma, int L, int Hkv, int D, int block_size, int max_blocks, int kv_dtype,
                       int br_dtype, void *k_cache, void *v_cache, const int32_t *block_tables,
                       const int32_t *prefix_lens, const void *k_branch, const void *v_branch, int C,
                       const void *k_pool, const void *v_pool, const int32_t *pool_seg, const uint64_t *commit_mask,
                       const int32_t *src_branch, const int32_t *n_own, const float *k_scale, const float *v_scale,
                       int32_t *new_prefix_lens) {
  if (B < 1 || gamma < 1 || L < 1 || Hkv < 1 || D < 1 || block_size < 1 || C < 0) return 1;
  if (!k_cache || !v_cache || !prefix_lens || !k_branch || !v_branch || !src_branch || !commit_mask || !n_own ||
      !new_prefix_lens)
    return 1;
  if (C > 0 && (!k_pool || !v_pool || !pool_seg)) return 1;
  for (int64_t i = 0; i < (int64_t)B * C; ++i)
    if (pool_seg[i] < 0 || pool_seg[i] > 63) return 1;
  int *rows = (int *)malloc(sizeof(int) * (size_t)(C > 0 ? C : 1));
  if (!rows) return 3;
  int rc = 0;
  for (int b = 0; b < B && !rc; ++b) {
    int kept = 0;
    for (int c = 0; c < C; ++c)
      if ((commit_mask[b] >> pool_seg[(int64_t)b * C + c]) & 1u) rows[kept++] = c;
    if (src_branch[b] < 0 || src_branch[b] >= gamma || n_own[b] < 0 || n_own[b] > L ||
        (int64_t)prefix_lens[b] + kept + n_own[b] > (int64_t)max_blocks * block_size) {
      rc = 1;
      break;
    }
    rc = commit_request(b, gamma, L, Hkv, D, block_size, max_blocks, kv_dtype, br_dtype, k_cache, v_cache,
                        block_tables, prefix_lens[b], k_branch, v_branch, C, k_pool, v_pool, rows, kept,
                        src_branch[b], n_own[b], k_scale, v_scale);
    new_prefix_lens[b] = prefix_lens[b] + kept + n_own[b];
  }
  free(rows);
  return rc;
}

/* Test hook: the quantiser alone, n fp32 values divided by `scale`. */
int lao_quantize_fp8_e4m3(const float *x, int64_t n, float scale, uint8_t *codes) {
  if (!x || !codes || !(scale > 0.0f)) return 1;
  for (int64_t i = 0; i < n; ++i) codes[i] = nearest_fp8_e4m3fn(x[i] / scale);
  return 0;
}

#ifdef _OPENMP
#include <omp.h>
int lao_num_threads(void) { return omp_get_max_threads(); }
#else
int lao_num_threads(void) { return 1; }
#endif
