// Host side of libla_verify: argument validation, launch planning, the extern "C" entry points
// declared in la_verify.h and the optional per-kernel event timing.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "la_internal.hpp"
#include <cstdio>

namespace la {
namespace {

constexpr int kNumCUs = 256;  // MI355X

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }
inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

enum AttnPath { PATH_NONE = 0, PATH_F32, PATH_MFMA };

struct AttnPlan {
  AttnPath path;
  bool kv_fp8, br_fp8;
  int shape, tile_m, n_row_tiles, chunk_len, s_max, total_units;
  size_t part_o_bytes, part_ml_bytes;
};

la_status validate_desc(const la_attn_desc *d) {
  if (!d) return LA_ERR_INVALID_ARG;
  if (d->num_requests < 1 || d->num_q_heads < 1 || d->num_kv_heads < 1 || d->head_dim < 1 || d->gamma < 1 ||
      d->branch_len < 1)
    return LA_ERR_INVALID_ARG;
  if (d->num_q_heads % d->num_kv_heads) return LA_ERR_INVALID_ARG;
  if (d->block_size < 16 || (d->block_size & (d->block_size - 1))) return LA_ERR_INVALID_ARG;  // power of two
  if (d->max_blocks_per_request < 0) return LA_ERR_INVALID_ARG;
  if (!(d->softmax_scale > 0.f) || !isfinite(d->softmax_scale)) return LA_ERR_INVALID_ARG;
  if (d->kv_split_tokens < 0 || d->kv_split_tokens % 64) return LA_ERR_INVALID_ARG;
  const int32_t dts[4] = {d->q_dtype, d->kv_dtype, d->branch_kv_dtype, d->out_dtype};
  for (int i = 0; i < 4; ++i)
    if (dts[i] < LA_F32 || dts[i] > LA_FP8_E4M3) return LA_ERR_INVALID_ARG;
  // rows and prefix tokens are indexed with 32-bit integers on the device
  const int64_t n_rows = (int64_t)d->gamma * d->branch_len * d->num_q_heads;
  if (n_rows * d->num_requests > (int64_t)1 << 30) return LA_ERR_UNSUPPORTED;
  if ((int64_t)d->max_blocks_per_request * d->block_size > (int64_t)1 << 30) return LA_ERR_UNSUPPORTED;
  return LA_OK;
}

la_status make_plan(const la_attn_desc *d, const int32_t *prefix_lens_host, AttnPlan *plan) {
  la_status st = validate_desc(d);
  if (st != LA_OK) return st;
  if (!prefix_lens_host) return LA_ERR_INVALID_ARG;
  int64_t max_p = 0;
  for (int b = 0; b < d->num_requests; ++b) {
    const int64_t P = prefix_lens_host[b];
    if (P < 0 || P > (int64_t)d->max_blocks_per_request * d->block_size) return LA_ERR_INVALID_ARG;
    max_p = P > max_p ? P : max_p;
  }
  memset(plan, 0, sizeof *plan);
  const bool all_f32 =
      d->q_dtype == LA_F32 && d->kv_dtype == LA_F32 && d->branch_kv_dtype == LA_F32 && d->out_dtype == LA_F32;
  if (all_f32) {
    if (d->head_dim != 64 && d->head_dim != 128 && d->head_dim != 256) return LA_ERR_UNSUPPORTED;
    plan->path = PATH_F32;
    return LA_OK;
  }
  const bool out_ok = d->out_dtype == LA_BF16 || d->out_dtype == LA_F32;
  const bool bf16_all = d->q_dtype == LA_BF16 && d->kv_dtype == LA_BF16 && d->branch_kv_dtype == LA_BF16;
  const bool fp8_kv = d->q_dtype == LA_BF16 && d->kv_dtype == LA_FP8_E4M3 &&
                      (d->branch_kv_dtype == LA_FP8_E4M3 || d->branch_kv_dtype == LA_BF16);
  if (!out_ok || !(bf16_all || fp8_kv) || d->head_dim != 128) return LA_ERR_UNSUPPORTED;
  plan->path = PATH_MFMA;
  plan->kv_fp8 = d->kv_dtype == LA_FP8_E4M3;
  plan->br_fp8 = d->branch_kv_dtype == LA_FP8_E4M3;

  const int G = d->num_q_heads / d->num_kv_heads;
  const int R = d->gamma * d->branch_len * G;
  const size_t n_rows = (size_t)d->gamma * d->branch_len * d->num_q_heads;

  // Choose the kernel shape and the chunk length that minimise a simple cost model (microseconds, constants
  // fitted to measurements on MI355X):
  //   rounds of workgroups over the CU slots  x  (tiles per chunk x time per 64-key tile + fixed start-up)
  //   + the merge of the partials (rows x (D+2) floats per chunk, written once and read once).
  // Few long chunks keep the partial traffic small, many short ones fill the chip when there are few rows.
  // Candidates: the 256-row shape (one workgroup per CU) and the 128-row two-stage shape (two per CU).
  const int candidates[2] = {0, 1};
  int forced = -1;
  if (const char *e = getenv("LA_ATTN_SHAPE")) {  // tuning override: index into the kernel's shape table
    const int v = atoi(e);
    if (v >= 0 && v < attn_mfma_num_shapes()) forced = v;
  }
  double best_cost = 0.0;
  int best_len = 0, best_shape = -1;
  for (int ci = 0; ci < (forced >= 0 ? 1 : 2); ++ci) {
    const int shape = forced >= 0 ? forced : candidates[ci];
    const int tile_m = attn_mfma_tile_m(shape);
    const int per_cu = attn_mfma_wgs_per_cu(shape);
    const int64_t base_wgs = (int64_t)d->num_kv_heads * ((R + tile_m - 1) / tile_m);
    const double t_tile = per_cu > 1 ? 2.25 : 1.87;  // per workgroup and 64-key tile, the CU shared by per_cu
    const double t_fixed = per_cu > 1 ? 8.0 : 9.0;
    // the workgroup of a request's last chunk also runs the branch-private tiles (masked, not pipelined: about
    // three times the cost of a prefix tile each), so the last chunk is made that much shorter than the others
    const int priv_tokens = tile_m / G + d->branch_len < d->gamma * d->branch_len ? tile_m / G + d->branch_len
                                                                                 : d->gamma * d->branch_len;
    const int64_t extra_tiles = 3 * (int64_t)((priv_tokens + 63) / 64);
    for (int n = 1; n <= 512; ++n) {
      int64_t len = max_p > 0 ? (max_p + (n > 1 ? extra_tiles * 64 : 0) + n - 1) / n : 64;
      len = ((len + 63) / 64) * 64;
      if (d->kv_split_tokens) len = d->kv_split_tokens;
      int64_t units = 0;
      for (int b = 0; b < d->num_requests; ++b) units += attn_num_chunks(prefix_lens_host[b], (int)len);
      const int64_t slots = (int64_t)kNumCUs * per_cu;
      const int64_t rounds = (base_wgs * units + slots - 1) / slots;
      const double merge_us = 3.0 + (double)units * n_rows * (d->head_dim + 2) * 4.0 / 3.0e6;  // read at ~3 TB/s
      const int64_t n_max = attn_num_chunks((int)max_p, (int)len);
      const int64_t last_tiles = (max_p - (n_max - 1) * len + 63) / 64 + extra_tiles;  // of the longest request
      const int64_t wg_tiles = n_max > 1 && len / 64 > last_tiles ? len / 64 : last_tiles;
      const double cost = (double)rounds * ((double)wg_tiles * t_tile + t_fixed) + merge_us;
      if (best_shape < 0 || cost < best_cost) best_cost = cost, best_len = (int)len, best_shape = shape;
      if (len <= 64 || d->kv_split_tokens) break;
    }
  }
  plan->shape = best_shape;
  plan->tile_m = attn_mfma_tile_m(plan->shape);
  plan->n_row_tiles = (R + plan->tile_m - 1) / plan->tile_m;
  int chunk = best_len;
  // the block ids of one chunk live in LDS
  const int64_t max_chunk = (int64_t)(attn_mfma_max_chunk_blocks() - 1) * d->block_size;  // -1: unaligned chunk start
  if (chunk > max_chunk) {
    if (d->kv_split_tokens) return LA_ERR_UNSUPPORTED;
    chunk = (int)(max_chunk / 64 * 64);
  }
  plan->chunk_len = chunk;
  int s_max = 1, total = 0;
  for (int b = 0; b < d->num_requests; ++b) {
    const int nc = attn_num_chunks(prefix_lens_host[b], chunk);
    s_max = nc > s_max ? nc : s_max;
    total += nc;
  }
  plan->s_max = s_max;
  plan->total_units = total;
  plan->part_o_bytes = align_up((size_t)d->num_requests * s_max * n_rows * d->head_dim * sizeof(float));
  plan->part_ml_bytes = align_up((size_t)d->num_requests * s_max * n_rows * 2 * sizeof(float));
  if (getenv("LA_DEBUG_PLAN"))
    fprintf(stderr, "la plan: shape %d (tile_m %d) row_tiles %d chunk_len %d units %d s_max %d\n", plan->shape,
            plan->tile_m, plan->n_row_tiles, plan->chunk_len, plan->total_units, plan->s_max);
  return LA_OK;
}

// ---- profiling ---------------------------------------------------------------------------------
const char *kSlotNames[SLOT_COUNT] = {"attn_mfma",     "attn_merge",   "attn_f32",   "accept_stats", "accept_warp",
                                      "accept_decide", "accept_resid", "accept_pick", "kv_commit",
                                      "calib_mfma",    "calib_read"};
struct ProfileRecord {
  int slot;
  hipEvent_t start, stop;
};
bool g_profile_on = false;
uint32_t g_profile_mask = 0xffffffffu;      // slots that are timed
int g_profile_stride = 1;                   // of their launches, every stride-th one
int64_t g_seen[SLOT_COUNT];                 // launches of a slot seen while enabled
std::vector<ProfileRecord> g_records;       // pending (not yet collected)
std::vector<hipEvent_t> g_free_events;
int64_t g_launches[SLOT_COUNT];
double g_total_ms[SLOT_COUNT];
hipEvent_t g_open_start;                    // start event of the scope being recorded
bool g_open = false;

hipEvent_t take_event() {
  if (!g_free_events.empty()) {
    hipEvent_t e = g_free_events.back();
    g_free_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

}  // namespace

void profile_before(int slot, hipStream_t stream) {
  g_open = false;
  if (!g_profile_on || !((g_profile_mask >> slot) & 1u)) return;
  if ((g_seen[slot]++ % g_profile_stride) != 0 || g_records.size() >= LA_PROFILE_MAX_RECORDS) return;
  hipEvent_t e = take_event();
  if (!e) return;
  if (hipEventRecord(e, stream) != hipSuccess) {
    g_free_events.push_back(e);
    return;
  }
  g_open_start = e;
  g_open = true;
}

void profile_after(int slot, hipStream_t stream) {
  if (!g_open) return;
  g_open = false;
  hipEvent_t e = take_event();
  if (!e || hipEventRecord(e, stream) != hipSuccess) {
    if (e) g_free_events.push_back(e);
    g_free_events.push_back(g_open_start);
    return;
  }
  g_records.push_back({slot, g_open_start, e});
}

}  // namespace la

using namespace la;

extern "C" {

const char *la_status_string(la_status s) {
  switch (s) {
    case LA_OK: return "ok";
    case LA_ERR_INVALID_ARG: return "invalid argument";
    case LA_ERR_UNSUPPORTED: return "unsupported shape or dtype combination";
    case LA_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case LA_ERR_LAUNCH: return "kernel launch failed";
  }
  return "unknown status";
}

la_status la_verify_attention_workspace(const la_attn_desc *desc, const int32_t *prefix_lens_host,
                                        size_t *bytes_out) {
  if (!bytes_out) return LA_ERR_INVALID_ARG;
  AttnPlan plan;
  la_status st = make_plan(desc, prefix_lens_host, &plan);
  if (st != LA_OK) return st;
  *bytes_out = plan.path == PATH_MFMA ? plan.part_o_bytes + plan.part_ml_bytes : 0;
  return LA_OK;
}

// Shared by the three attention entry points.  chain_len tokens of extra K/V per request: a chain with a visible
// leading part per branch (chain_vis), or a pool with segment labels and a segment mask per branch (pool_seg).
static la_status verify_attention(const la_attn_desc *desc, const void *q, const void *k_cache, const void *v_cache,
                                  const int32_t *block_tables, const int32_t *prefix_lens,
                                  const int32_t *prefix_lens_host, const void *k_branch, const void *v_branch,
                                  const void *k_chain, const void *v_chain, int32_t chain_len,
                                  const int32_t *chain_vis, const int32_t *chain_vis_host, const int32_t *pool_seg,
                                  const int32_t *pool_seg_host, const uint64_t *seg_mask, const float *k_scale,
                                  const float *v_scale, void *out, float *lse, void *workspace,
                                  size_t workspace_bytes, void *hip_stream) {
  AttnPlan plan;
  la_status st = make_plan(desc, prefix_lens_host, &plan);
  if (st != LA_OK) return st;
  if (!q || !prefix_lens || !k_branch || !v_branch || !out) return LA_ERR_INVALID_ARG;
  bool any_prefix = false;
  for (int b = 0; b < desc->num_requests; ++b) any_prefix |= prefix_lens_host[b] > 0;
  if (any_prefix && (!k_cache || !v_cache)) return LA_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(k_branch) || !aligned16(v_branch) ||
      !aligned16(out) || !aligned16(workspace))
    return LA_ERR_INVALID_ARG;
  if (chain_len < 0) return LA_ERR_INVALID_ARG;
  const bool tree = pool_seg != nullptr || pool_seg_host != nullptr || seg_mask != nullptr;
  if (chain_len > 0) {
    if (!k_chain || !v_chain || !aligned16(k_chain) || !aligned16(v_chain)) return LA_ERR_INVALID_ARG;
    if (tree) {
      if (!pool_seg || !pool_seg_host || !seg_mask || ((uintptr_t)seg_mask & 7)) return LA_ERR_INVALID_ARG;
      for (int64_t t = 0; t < (int64_t)desc->num_requests * chain_len; ++t)
        if (pool_seg_host[t] < 0 || pool_seg_host[t] > 63) return LA_ERR_INVALID_ARG;
    } else {
      if (!chain_vis || !chain_vis_host) return LA_ERR_INVALID_ARG;
      for (int64_t t = 0; t < (int64_t)desc->num_requests * desc->gamma; ++t)
        if (chain_vis_host[t] < 0 || chain_vis_host[t] > chain_len) return LA_ERR_INVALID_ARG;
    }
  }
  const size_t need = plan.path == PATH_MFMA ? plan.part_o_bytes + plan.part_ml_bytes : 0;
  if (need > 0 && (!workspace || workspace_bytes < need)) return LA_ERR_WORKSPACE_TOO_SMALL;

  AttnParams p;
  memset(&p, 0, sizeof p);
  p.q = q, p.k_cache = k_cache, p.v_cache = v_cache, p.k_branch = k_branch, p.v_branch = v_branch;
  p.k_chain = k_chain, p.v_chain = v_chain, p.chain_vis = chain_vis, p.C = chain_len;
  if (chain_len > 0 && tree) p.pool_seg = pool_seg, p.seg_mask = seg_mask;
  p.block_tables = block_tables, p.prefix_lens = prefix_lens;
  p.k_scale = k_scale, p.v_scale = v_scale;
  p.out = out, p.lse = lse;
  p.B = desc->num_requests, p.Hq = desc->num_q_heads, p.Hkv = desc->num_kv_heads;
  p.G = p.Hq / p.Hkv, p.D = desc->head_dim, p.gamma = desc->gamma, p.L = desc->branch_len;
  p.block_size = desc->block_size, p.max_blocks = desc->max_blocks_per_request;
  p.block_shift = __builtin_ctz((unsigned)desc->block_size);
  p.R = p.gamma * p.L * p.G;
  p.n_rows = p.gamma * p.L * p.Hq;
  p.out_f32 = desc->out_dtype == LA_F32;
  p.scale_log2 = desc->softmax_scale * 1.44269504088896340736f;
  hipStream_t stream = (hipStream_t)hip_stream;

  if (plan.path == PATH_F32) return launch_attn_f32(p, stream) == hipSuccess ? LA_OK : LA_ERR_LAUNCH;

  p.n_row_tiles = plan.n_row_tiles, p.chunk_len = plan.chunk_len, p.s_max = plan.s_max;
  p.total_units = plan.total_units;
  p.part_o = (float *)workspace;
  p.part_ml = (float *)((uint8_t *)workspace + plan.part_o_bytes);
  if (launch_attn_mfma(p, plan.shape, plan.kv_fp8, plan.br_fp8, stream) != hipSuccess) return LA_ERR_LAUNCH;
  if (launch_attn_merge(p, stream) != hipSuccess) return LA_ERR_LAUNCH;
  return LA_OK;
}

la_status la_verify_attention(const la_attn_desc *desc, const void *q, const void *k_cache, const void *v_cache,
                              const int32_t *block_tables, const int32_t *prefix_lens,
                              const int32_t *prefix_lens_host, const void *k_branch, const void *v_branch,
                              const float *k_scale, const float *v_scale, void *out, float *lse, void *workspace,
                              size_t workspace_bytes, void *hip_stream) {
  return verify_attention(desc, q, k_cache, v_cache, block_tables, prefix_lens, prefix_lens_host, k_branch, v_branch,
                          nullptr, nullptr, 0, nullptr, nullptr, nullptr, nullptr, nullptr, k_scale, v_scale, out, lse,
                          workspace, workspace_bytes, hip_stream);
}

la_status la_verify_attention_nested(const la_attn_desc *desc, const void *q, const void *k_cache,
                                     const void *v_cache, const int32_t *block_tables, const int32_t *prefix_lens,
                                     const int32_t *prefix_lens_host, const void *k_branch, const void *v_branch,
                                     const void *k_chain, const void *v_chain, int32_t chain_len,
                                     const int32_t *chain_vis, const int32_t *chain_vis_host, const float *k_scale,
                                     const float *v_scale, void *out, float *lse, void *workspace,
                                     size_t workspace_bytes, void *hip_stream) {
  return verify_attention(desc, q, k_cache, v_cache, block_tables, prefix_lens, prefix_lens_host, k_branch, v_branch,
                          k_chain, v_chain, chain_len, chain_vis, chain_vis_host, nullptr, nullptr, nullptr, k_scale,
                          v_scale, out, lse, workspace, workspace_bytes, hip_stream);
}

la_status la_verify_attention_tree(const la_attn_desc *desc, const void *q, const void *k_cache, const void *v_cache,
                                   const int32_t *block_tables, const int32_t *prefix_lens,
                                   const int32_t *prefix_lens_host, const void *k_branch, const void *v_branch,
                                   const void *k_pool, const void *v_pool, int32_t pool_len, const int32_t *pool_seg,
                                   const int32_t *pool_seg_host, const uint64_t *seg_mask, const float *k_scale,
                                   const float *v_scale, void *out, float *lse, void *workspace,
                                   size_t workspace_bytes, void *hip_stream) {
  if (pool_len > 0 && (!pool_seg || !pool_seg_host || !seg_mask)) return LA_ERR_INVALID_ARG;
  return verify_attention(desc, q, k_cache, v_cache, block_tables, prefix_lens, prefix_lens_host, k_branch, v_branch,
                          k_pool, v_pool, pool_len, nullptr, nullptr, pool_len > 0 ? pool_seg : nullptr,
                          pool_len > 0 ? pool_seg_host : nullptr, pool_len > 0 ? seg_mask : nullptr, k_scale, v_scale,
                          out, lse, workspace, workspace_bytes, hip_stream);
}

// Shared by la_kv_commit (pool_seg == nullptr: the first n_chain tokens of the chain are kept) and
// la_kv_commit_tree (the pool tokens whose node has its bit in commit_mask are kept; n_chain == nullptr).
static la_status kv_commit(const la_attn_desc *desc, void *k_cache, void *v_cache, const int32_t *block_tables,
                           const int32_t *prefix_lens, const int32_t *prefix_lens_host, const void *k_branch,
                           const void *v_branch, const void *k_chain, const void *v_chain, int32_t chain_len,
                           const int32_t *pool_seg, const uint64_t *commit_mask, const int32_t *src_branch,
                           const int32_t *n_chain, const int32_t *n_own, const float *k_scale, const float *v_scale,
                           int32_t *new_prefix_lens, const la_layer_strides *layers, void *hip_stream) {
  const bool tree = commit_mask != nullptr;
  la_status st = validate_desc(desc);
  if (st != LA_OK) return st;
  if (!k_cache || !v_cache || !prefix_lens || !prefix_lens_host || !k_branch || !v_branch || !src_branch ||
      (!tree && !n_chain) || !n_own || !new_prefix_lens)
    return LA_ERR_INVALID_ARG;
  if (new_prefix_lens == prefix_lens) return LA_ERR_INVALID_ARG;  // read by every workgroup while one writes
  if (chain_len < 0 || (chain_len > 0 && (!k_chain || !v_chain))) return LA_ERR_INVALID_ARG;
  if (tree && ((chain_len > 0 && !pool_seg) || ((uintptr_t)commit_mask & 7))) return LA_ERR_INVALID_ARG;
  if (!aligned16(k_cache) || !aligned16(v_cache) || !aligned16(k_branch) || !aligned16(v_branch) ||
      !aligned16(k_chain) || !aligned16(v_chain))
    return LA_ERR_INVALID_ARG;
  const int kv = desc->kv_dtype, br = desc->branch_kv_dtype;
  const bool quantise = kv == LA_FP8_E4M3 && br == LA_BF16;
  if (kv != br && !quantise) return LA_ERR_UNSUPPORTED;
  if (desc->head_dim % 16) return LA_ERR_UNSUPPORTED;
  const int64_t capacity = (int64_t)desc->max_blocks_per_request * desc->block_size;
  // what is appended is decided on the device; the block table must have room for the most it can be
  for (int b = 0; b < desc->num_requests; ++b)
    if (prefix_lens_host[b] < 0 || (int64_t)prefix_lens_host[b] + chain_len + desc->branch_len > capacity)
      return LA_ERR_INVALID_ARG;
  const int n_layers = layers ? layers->num_layers : 1;
  if (n_layers < 1 || n_layers > 65535 || desc->num_requests > 65535) return LA_ERR_INVALID_ARG;
  const int elem_bytes[3] = {4, 2, 1};  // LA_F32, LA_BF16, LA_FP8_E4M3
  if (layers) {
    if (layers->cache_stride < 0 || layers->branch_stride < 0 || layers->chain_stride < 0 ||
        layers->scale_stride < 0)
      return LA_ERR_INVALID_ARG;
    // every layer's tensors must start on a 16-byte boundary
    if ((layers->cache_stride * elem_bytes[kv]) % 16 || (layers->branch_stride * elem_bytes[br]) % 16 ||
        (layers->chain_stride * elem_bytes[br]) % 16)
      return LA_ERR_INVALID_ARG;
  }

  CommitParams p;
  memset(&p, 0, sizeof p);
  p.k_cache = k_cache, p.v_cache = v_cache;
  p.k_branch = k_branch, p.v_branch = v_branch, p.k_chain = k_chain, p.v_chain = v_chain;
  p.block_tables = block_tables, p.prefix_lens = prefix_lens;
  p.src_branch = src_branch, p.n_chain = n_chain, p.n_own = n_own;
  p.pool_seg = tree && chain_len > 0 ? pool_seg : nullptr;  // an empty pool is the chain form with nothing kept
  p.commit_mask = commit_mask;
  p.k_scale = k_scale, p.v_scale = v_scale;
  p.new_prefix_lens = new_prefix_lens;
  p.B = desc->num_requests, p.Hkv = desc->num_kv_heads, p.D = desc->head_dim, p.gamma = desc->gamma;
  p.L = desc->branch_len, p.C = chain_len;
  p.block_size = desc->block_size, p.block_shift = __builtin_ctz((unsigned)desc->block_size);
  p.max_blocks = desc->max_blocks_per_request;
  p.capacity = (int)capacity;
  p.num_layers = n_layers;
  if (layers) {
    p.cache_stride = layers->cache_stride, p.branch_stride = layers->branch_stride;
    p.chain_stride = layers->chain_stride, p.scale_stride = layers->scale_stride;
  }
  return launch_kv_commit(p, elem_bytes[br], quantise, (hipStream_t)hip_stream) == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

la_status la_kv_commit(const la_attn_desc *desc, void *k_cache, void *v_cache, const int32_t *block_tables,
                       const int32_t *prefix_lens, const int32_t *prefix_lens_host, const void *k_branch,
                       const void *v_branch, const void *k_chain, const void *v_chain, int32_t chain_len,
                       const int32_t *src_branch, const int32_t *n_chain, const int32_t *n_own, const float *k_scale,
                       const float *v_scale, int32_t *new_prefix_lens, const la_layer_strides *layers,
                       void *hip_stream) {
  if (!n_chain) return LA_ERR_INVALID_ARG;
  return kv_commit(desc, k_cache, v_cache, block_tables, prefix_lens, prefix_lens_host, k_branch, v_branch, k_chain,
                   v_chain, chain_len, nullptr, nullptr, src_branch, n_chain, n_own, k_scale, v_scale,
                   new_prefix_lens, layers, hip_stream);
}

la_status la_kv_commit_tree(const la_attn_desc *desc, void *k_cache, void *v_cache, const int32_t *block_tables,
                            const int32_t *prefix_lens, const int32_t *prefix_lens_host, const void *k_branch,
                            const void *v_branch, const void *k_pool, const void *v_pool, int32_t pool_len,
                            const int32_t *pool_seg, const uint64_t *commit_mask, const int32_t *src_branch,
                            const int32_t *n_own, const float *k_scale, const float *v_scale,
                            int32_t *new_prefix_lens, const la_layer_strides *layers, void *hip_stream) {
  if (!commit_mask) return LA_ERR_INVALID_ARG;
  return kv_commit(desc, k_cache, v_cache, block_tables, prefix_lens, prefix_lens_host, k_branch, v_branch, k_pool,
                   v_pool, pool_len, pool_seg, commit_mask, src_branch, nullptr, n_own, k_scale, v_scale,
                   new_prefix_lens, layers, hip_stream);
}

static la_status validate_accept(const la_accept_desc *d) {
  if (!d) return LA_ERR_INVALID_ARG;
  if (d->num_branches < 1 || d->num_draft < 1 || d->vocab < 1) return LA_ERR_INVALID_ARG;
  if (d->top_k < 0 || !(d->top_p > 0.0f) || d->top_p > 1.0f) return LA_ERR_INVALID_ARG;
  if (d->logits_dtype != LA_F32 && d->logits_dtype != LA_BF16)
    return d->logits_dtype == LA_FP8_E4M3 ? LA_ERR_UNSUPPORTED : LA_ERR_INVALID_ARG;
  if (!(d->temperature > 0.f) || !isfinite(d->temperature)) return LA_ERR_INVALID_ARG;
  if ((int64_t)d->num_branches * (2 * (int64_t)d->num_draft + 1) > 65535) return LA_ERR_UNSUPPORTED;  // grid.y
  if (d->vocab > (1 << 21)) return LA_ERR_UNSUPPORTED;  // fine slices of one row are staged in LDS
  return LA_OK;
}

la_status la_selftest_exp64(const double *y, double *out, size_t n, void *hip_stream) {
  if (!y || !out || n < 1 || n > ((size_t)1 << 30)) return LA_ERR_INVALID_ARG;
  return launch_exp64_probe(y, out, n, (hipStream_t)hip_stream) == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

la_status la_spec_accept_workspace(const la_accept_desc *desc, size_t *bytes_out) {
  la_status st = validate_accept(desc);
  if (st != LA_OK) return st;
  if (!bytes_out) return LA_ERR_INVALID_ARG;
  *bytes_out = accept_workspace_bytes(desc->num_branches, desc->num_draft, desc->vocab,
                                      desc->logits_dtype == LA_BF16, nullptr, nullptr);
  return LA_OK;
}

la_status la_spec_accept(const la_accept_desc *desc, const void *target_logits, const void *draft_logits,
                         const int32_t *draft_tokens, const float *u_accept, const float *u_sample,
                         int32_t *accepted_len, int32_t *next_token, float *accept_ratio, void *workspace,
                         size_t workspace_bytes, void *hip_stream) {
  la_status st = validate_accept(desc);
  if (st != LA_OK) return st;
  if (!target_logits || !draft_tokens || !u_accept || !u_sample || !accepted_len || !next_token)
    return LA_ERR_INVALID_ARG;
  if (!aligned16(target_logits) || (draft_logits && !aligned16(draft_logits)) || !aligned16(workspace))
    return LA_ERR_INVALID_ARG;
  AcceptParams p;
  memset(&p, 0, sizeof p);
  const size_t need = accept_workspace_bytes(desc->num_branches, desc->num_draft, desc->vocab,
                                             desc->logits_dtype == LA_BF16, &p.n_chunks, &p.n_fine);
  if (!workspace || workspace_bytes < need) return LA_ERR_WORKSPACE_TOO_SMALL;
  p.target = target_logits, p.draft = draft_logits, p.tokens = draft_tokens;
  p.u_accept = u_accept, p.u_sample = u_sample;
  p.accepted_len = accepted_len, p.next_token = next_token, p.ratio = accept_ratio;
  p.NB = desc->num_branches, p.K = desc->num_draft, p.V = desc->vocab;
  p.bf16 = desc->logits_dtype == LA_BF16;
  p.inv_temp_log2 = 1.44269504088896340736f / desc->temperature;
  p.inv_temp = 1.0 / (double)desc->temperature;
  p.top_k = desc->top_k, p.top_p = desc->top_p;
  accept_carve_workspace(p, workspace);
  return launch_accept(p, (hipStream_t)hip_stream) == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

la_status la_profile_select(uint32_t slot_mask, int32_t stride) {
  if (stride < 1) return LA_ERR_INVALID_ARG;
  g_profile_mask = slot_mask;
  g_profile_stride = stride;
  return LA_OK;
}

la_status la_profile_enable(int on) {
  g_profile_on = on != 0;
  return LA_OK;
}

la_status la_profile_collect(void) {
  la_status st = LA_OK;
  for (const ProfileRecord &r : g_records) {
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) == hipSuccess && hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
      g_launches[r.slot] += 1;
      g_total_ms[r.slot] += ms;
    } else {
      st = LA_ERR_LAUNCH;
    }
    g_free_events.push_back(r.start);
    g_free_events.push_back(r.stop);
  }
  g_records.clear();
  return st;
}

int32_t la_profile_num_kernels(void) { return SLOT_COUNT; }

la_status la_profile_get(int32_t slot, const char **name, int64_t *launches, double *total_ms) {
  if (slot < 0 || slot >= SLOT_COUNT) return LA_ERR_INVALID_ARG;
  if (name) *name = kSlotNames[slot];
  if (launches) *launches = g_launches[slot];
  if (total_ms) *total_ms = g_total_ms[slot];
  return LA_OK;
}

la_status la_profile_reset(void) {
  la_status st = la_profile_collect();
  for (int i = 0; i < SLOT_COUNT; ++i) g_launches[i] = 0, g_total_ms[i] = 0.0, g_seen[i] = 0;
  return st;
}

}  // extern "C"
