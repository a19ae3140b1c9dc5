// Host side of libla_verify: argument validation, launch planning, the extern "C" entry points
// declared in la_verify.h and the optional per-kernel event timing.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include "la_internal.hpp"
#include <cstdio>

namespace la {
namespace {

// Compute units of the current device, asked once (256 on MI355X, also the fallback when no device answers, e.g. a
// workspace query on a machine without a GPU).
int num_cus() {
  static std::once_flag once;
  static int cus = 256;
  std::call_once(once, [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
  });
  return cus;
}

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }
inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

enum AttnPath { PATH_NONE = 0, PATH_F32, PATH_MFMA };

// Kernel shapes of the MFMA path, numbered as la_attn_desc.kernel_shape - 1 numbers them: the row-tile shapes of
// attn_mfma_kernel first, then the streaming shapes of attn_stream_kernel.
struct ShapeInfo {
  bool stream;
  bool fp8;        // streaming shapes: storage type of cache and branch K/V the shape is built for
  int local;       // index inside its kernel's own shape table
  int tile_m;      // query rows per workgroup
  int per_cu;      // workgroups that share a CU
  int step_keys;   // keys a workgroup advances per pipeline step
  double t_step;   // microseconds per step of one workgroup with the CU shared by per_cu (fitted)
  double t_step_shared;  // the same when several row tiles stream the same keys (streaming shapes: arithmetic-bound
                         // steps; with one row tile a step is bound by its share of the HBM stream)
  double t_fixed;  // microseconds of start-up and write-out per workgroup (fitted)
};
int num_shapes() { return attn_mfma_num_shapes() + attn_stream_num_shapes(); }
ShapeInfo shape_info(int shape) {
  ShapeInfo s{};
  if (shape < attn_mfma_num_shapes()) {
    s.stream = false, s.local = shape;
    s.tile_m = attn_mfma_tile_m(shape), s.per_cu = attn_mfma_wgs_per_cu(shape), s.step_keys = 64;
    s.t_step = s.t_step_shared = s.per_cu > 1 ? 2.25 : 1.87;
    s.t_fixed = s.per_cu > 1 ? 8.0 : 9.0;
  } else {
    s.stream = true, s.local = shape - attn_mfma_num_shapes();
    s.tile_m = attn_stream_tile_m(s.local), s.per_cu = 1;
    s.step_keys = attn_stream_step_keys(s.local);
    // every wavefront reduces one 64-key tile for its 32 rows per step, whatever the shape: the time of a step is
    // the time of two such units on one SIMD
    s.fp8 = attn_stream_shape_is_fp8(s.local);
    if (s.fp8) {
      s.t_step = s.tile_m == 64 ? 3.1 : s.tile_m == 128 ? 2.3 : 3.0;
      s.t_step_shared = s.tile_m == 64 ? 2.15 : s.tile_m == 128 ? 2.05 : 2.2;
    } else {
      s.t_step = s.t_step_shared = s.tile_m == 256 ? 1.8 : 2.45;
    }
    // (the 256-row bf16 shape: eight row blocks' Q into registers and a branch-private tile per wavefront at the end)
    s.t_fixed = (!s.fp8 && s.tile_m == 256) ? 12.0 : 5.0;
  }
  return s;
}

struct AttnPlan {
  AttnPath path;
  bool kv_fp8, br_fp8;
  int shape, tile_m, n_row_tiles, chunk_len, last_short, s_max, total_units;
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
  if (d->kernel_shape < 0 || d->kernel_shape > num_shapes()) return LA_ERR_INVALID_ARG;
  const int32_t dts[4] = {d->q_dtype, d->kv_dtype, d->branch_kv_dtype, d->out_dtype};
  for (int i = 0; i < 4; ++i)
    if (dts[i] < LA_F32 || dts[i] > LA_FP8_E4M3) return LA_ERR_INVALID_ARG;
  // rows and prefix tokens are indexed with 32-bit integers on the device
  const int64_t n_rows = (int64_t)d->gamma * d->branch_len * d->num_q_heads;
  if (n_rows * d->num_requests > (int64_t)1 << 30) return LA_ERR_UNSUPPORTED;
  if ((int64_t)d->max_blocks_per_request * d->block_size > (int64_t)1 << 30) return LA_ERR_UNSUPPORTED;
  return LA_OK;
}

// extra: the call carries a drafted chain or pool (nested / tree form)
la_status make_plan(const la_attn_desc *d, const int32_t *prefix_lens_host, bool extra, AttnPlan *plan) {
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
  if (!out_ok || !(bf16_all || fp8_kv)) return LA_ERR_UNSUPPORTED;
  if (d->head_dim != 128) {
    // the MFMA and streaming kernels are written for head dimension 128; 64 and 256 run on the general kernel
    // (fp32 arithmetic on exactly widened inputs, one wavefront per query row)
    if (d->head_dim != 64 && d->head_dim != 256) return LA_ERR_UNSUPPORTED;
    if (d->kernel_shape > 0) return LA_ERR_UNSUPPORTED;
    plan->path = PATH_F32;
    return LA_OK;
  }
  plan->path = PATH_MFMA;
  plan->kv_fp8 = d->kv_dtype == LA_FP8_E4M3;
  plan->br_fp8 = d->branch_kv_dtype == LA_FP8_E4M3;

  const int G = d->num_q_heads / d->num_kv_heads;
  const int R = d->gamma * d->branch_len * G;
  const size_t n_rows = (size_t)d->gamma * d->branch_len * d->num_q_heads;
  // the streaming shapes exist for flat calls with cache and branch K/V of one storage type
  auto stream_ok = [&](const ShapeInfo &si) {
    return !extra && plan->kv_fp8 == si.fp8 && plan->br_fp8 == si.fp8 &&
           (int64_t)d->num_kv_heads * d->block_size * d->head_dim * (si.fp8 ? 1 : 2) < ((int64_t)1 << 32);
  };
  if (d->kernel_shape > 0) {
    const ShapeInfo forced = shape_info(d->kernel_shape - 1);
    if (forced.stream && !stream_ok(forced)) return LA_ERR_UNSUPPORTED;
  }

  // Choose the kernel shape and the number of chunks that minimise a simple cost model (microseconds, constants
  // fitted to measurements on MI355X):
  //   rounds of workgroups over the CU slots  x  (steps per chunk x time per step + fixed start-up)
  //   + the merge of the partials (rows x (D+2) floats per chunk, written once and read once).
  // Few long chunks keep the partial traffic small, many short ones fill the chip when there are few rows.
  // A request's key tiles are dealt out evenly over its chunks (attn_chunk_range); the workgroup of the last chunk
  // also runs the branch-private tiles (masked, general form: about three prefix tiles each in the row-tile
  // shapes, whole pipeline steps in the streaming shapes), which count as `last_short` tiles of its share.
  double best_cost = 0.0;
  int best_len = 0, best_shape = -1, best_short = 0;
  const int64_t T = (max_p + 63) / 64;
  for (int shape = 0; shape < num_shapes(); ++shape) {
    if (d->kernel_shape > 0 && shape != d->kernel_shape - 1) continue;
    const ShapeInfo si = shape_info(shape);
    if (si.stream && !stream_ok(si)) continue;
    const int64_t base_wgs = (int64_t)d->num_kv_heads * ((R + si.tile_m - 1) / si.tile_m);
    const int priv_tokens = si.tile_m / G + d->branch_len < d->gamma * d->branch_len ? si.tile_m / G + d->branch_len
                                                                                     : d->gamma * d->branch_len;
    // (a streaming shape advances whole steps: the private tiles are steps of their own, so the last chunk gets as
    // many prefix steps fewer, or its workgroup would finish a step after all the others)
    const int priv_tiles = (priv_tokens + 63) / 64, step_tiles = si.step_keys / 64;
    const int last_short = si.stream ? step_tiles * ((priv_tiles + step_tiles - 1) / step_tiles) : 3 * priv_tiles;
    const int64_t slots = (int64_t)num_cus() * si.per_cu;
    // the block ids of one chunk live in LDS (-2: a chunk need not start on a block boundary)
    const int blk_cap = si.stream ? attn_stream_max_chunk_blocks() : attn_mfma_max_chunk_blocks();
    const int64_t max_chunk = ((int64_t)(blk_cap - 2) * d->block_size - 64 * (last_short + 2)) / 64 * 64;
    if (max_chunk < 64 || d->kv_split_tokens > max_chunk) continue;
    double prev_cost = 0.0;
    for (int n = 1; n <= 512; ++n) {
      int64_t len = max_p > 0 ? (max_p + n - 1) / n : 64;
      len = ((len + 63) / 64) * 64;
      if (len > max_chunk) len = max_chunk;
      if (d->kv_split_tokens) len = d->kv_split_tokens;
      int64_t units = 0;
      for (int b = 0; b < d->num_requests; ++b) units += attn_num_chunks(prefix_lens_host[b], (int)len);
      const int64_t rounds = (base_wgs * units + slots - 1) / slots;
      const double merge_us = 3.0 + (double)units * n_rows * (d->head_dim + 2) * 4.0 / 3.0e6;  // read at ~3 TB/s
      const int64_t n_max = attn_num_chunks((int)max_p, (int)len);
      const int64_t wg_tiles = (T + last_short + n_max - 1) / n_max;  // of the longest request
      const int64_t wg_steps = (wg_tiles * 64 + si.step_keys - 1) / si.step_keys;
      const double t_step = R > si.tile_m ? si.t_step_shared : si.t_step;
      // (an fp8 streaming plan of several rounds has measured at its model cost, the row-tile shapes it competes with there
      // -- partly filled row tiles of 256 rows -- below theirs: the margin keeps those cases with the row tiles)
      double busy_us = (double)rounds * ((double)wg_steps * t_step + si.t_fixed);
      if (d->num_requests > 1 && rounds > 1 && n <= 8 && units <= 64) {
        // Several requests of different lengths in several rounds, few chunks each: rounds x the longest chunk is
        // what the dispatch of equal workgroups gives; with unequal ones the workgroups are dealt out here as the
        // hardware deals them, in launch order (all workgroups of a chunk, chunk after chunk, request after request),
        // each to the slot that is free first.  (Measured at configuration 4's ragged batch: one chunk per request,
        // 1.17 ms; chunks of 8192 keys, 1.04 ms, where rounds x longest saw the two as equal.)  With many chunks per
        // request they are nearly equal and the simple form holds; every call plans, so this stays small (fixed
        // arrays, at most 64 chunks).
        constexpr int kCap = 256;
        struct Free { double t; int64_t n; };
        Free cur[kCap], nxt[kCap], mrg[kCap];
        int n_cur = 1;
        cur[0] = {0.0, slots};
        bool fits = true;
        for (int b = 0; b < d->num_requests && fits; ++b) {
          const int64_t nc = attn_num_chunks(prefix_lens_host[b], (int)len);
          const int64_t tiles_b = (prefix_lens_host[b] + 63) / 64 + last_short;
          for (int64_t c = 0; c < nc && fits; ++c) {
            const int64_t tiles = tiles_b / nc + (c < tiles_b % nc ? 1 : 0);
            const double dur = (double)((tiles * 64 + si.step_keys - 1) / si.step_keys) * t_step + si.t_fixed;
            for (int64_t left = base_wgs; left > 0 && fits;) {
              int64_t need = left < slots ? left : slots;  // (the entries always add up to `slots`)
              left -= need;
              int i = 0, n_nxt = 0;
              for (; need > 0 && i < n_cur; ++i) {
                const int64_t k = need < cur[i].n ? need : cur[i].n;
                nxt[n_nxt++] = {cur[i].t + dur, k};
                cur[i].n -= k, need -= k;
                if (cur[i].n > 0) break;
              }
              // what was not taken keeps its place; the slots just filled come free later, in the order taken
              int a2 = i, b2 = 0, n_mrg = 0;
              while (a2 < n_cur || b2 < n_nxt) {
                if (n_mrg >= kCap) {
                  fits = false;
                  break;
                }
                if (b2 >= n_nxt || (a2 < n_cur && cur[a2].t <= nxt[b2].t)) {
                  if (cur[a2].n > 0) mrg[n_mrg++] = cur[a2];
                  ++a2;
                } else {
                  mrg[n_mrg++] = nxt[b2++];
                }
              }
              if (n_mrg + 2 >= kCap) fits = false;
              for (int j = 0; j < n_mrg; ++j) cur[j] = mrg[j];
              n_cur = n_mrg;
            }
          }
        }
        if (fits && n_cur > 0) busy_us = cur[n_cur - 1].t;
      }
      // (an fp8 streaming plan of several rounds has measured at its model cost, the row-tile shapes it competes with there
      // -- partly filled row tiles of 256 rows -- below theirs: the margin keeps those cases with the row tiles)
      const double cost = busy_us * (si.stream && si.fp8 && rounds > 1 ? 1.06 : 1.0) + merge_us;
      if (best_shape < 0 || cost < best_cost)
        best_cost = cost, best_len = (int)len, best_shape = shape, best_short = last_short;
      if (len <= 64 || d->kv_split_tokens) break;
      // once every slot is used and the cost has started to rise, more chunks only add partials
      if (n > 1 && rounds > 1 && cost > prev_cost && base_wgs * units > 4 * slots) break;
      prev_cost = cost;
    }
  }
  if (best_shape < 0) return LA_ERR_UNSUPPORTED;
  const ShapeInfo si = shape_info(best_shape);
  plan->shape = best_shape;
  plan->tile_m = si.tile_m;
  plan->n_row_tiles = (R + plan->tile_m - 1) / plan->tile_m;
  const int chunk = best_len;
  plan->chunk_len = chunk;
  plan->last_short = best_short;
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
  return LA_OK;
}

}  // namespace

}  // namespace la

using namespace la;

extern "C" {

const char *la_status_string(int32_t status) {
  switch (status) {
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
  // one size serves the flat, nested and tree calls (their plans may differ)
  size_t bytes = 0;
  for (int extra = 0; extra < 2; ++extra) {
    AttnPlan plan;
    la_status st = make_plan(desc, prefix_lens_host, extra != 0, &plan);
    if (extra && st == LA_ERR_UNSUPPORTED) continue;  // a forced shape that only runs flat calls
    if (st != LA_OK) return st;
    const size_t need = plan.path == PATH_MFMA ? plan.part_o_bytes + plan.part_ml_bytes : 0;
    bytes = need > bytes ? need : bytes;
  }
  *bytes_out = bytes;
  return LA_OK;
}

la_status la_verify_attention_plan(const la_attn_desc *desc, const int32_t *prefix_lens_host, int32_t chain_len,
                                   la_attn_plan *out) {
  if (!out || chain_len < 0) return LA_ERR_INVALID_ARG;
  AttnPlan plan;
  la_status st = make_plan(desc, prefix_lens_host, chain_len > 0, &plan);
  if (st != LA_OK) return st;
  memset(out, 0, sizeof *out);
  out->path = (int32_t)plan.path;
  if (plan.path == PATH_MFMA) {
    out->kernel_shape = plan.shape + 1;
    out->rows_per_workgroup = plan.tile_m;
    out->row_tiles = plan.n_row_tiles;
    out->chunk_tokens = plan.chunk_len;
    out->chunks_total = plan.total_units;
    out->workgroups = desc->num_kv_heads * plan.n_row_tiles * plan.total_units;
  }
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
  la_status st = make_plan(desc, prefix_lens_host, chain_len > 0, &plan);
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
  p.q_type = desc->q_dtype, p.kv_type = desc->kv_dtype, p.br_type = desc->branch_kv_dtype;
  p.scale_log2 = desc->softmax_scale * 1.44269504088896340736f;
  hipStream_t stream = (hipStream_t)hip_stream;

  if (plan.path == PATH_F32) return launch_attn_f32(p, stream) == hipSuccess ? LA_OK : LA_ERR_LAUNCH;

  p.n_row_tiles = plan.n_row_tiles, p.chunk_len = plan.chunk_len, p.s_max = plan.s_max;
  p.last_short = plan.last_short;
  p.total_units = plan.total_units;
  p.part_o = (float *)workspace;
  p.part_ml = (float *)((uint8_t *)workspace + plan.part_o_bytes);
  if (p.B <= kMaxInlineLens) {
    p.n_inline = p.B;
    for (int b = 0; b < p.B; ++b) {
      AttnParams::Req &rq = p.req[b];
      rq.P = prefix_lens_host[b];
      rq.n = attn_num_chunks(rq.P, p.chunk_len);
      const int64_t tv = ((int64_t)rq.P + 63) / 64 + p.last_short;
      rq.q = (int)(tv / rq.n), rq.r = (int)(tv % rq.n);
      // n == 1: r == 0, the quotient is never needed.  The multiply-shift is exact for x < 2^32 / n; the kernel
      // applies it to x <= n * r < n^2, so very many chunks take the kernel's general path instead.
      rq.inv = rq.n > 1 ? (uint32_t)(((uint64_t)1 << 32) / (uint64_t)rq.n) + 1u : 0u;
      if (rq.n > 1024) p.n_inline = 0;
    }
  }
  const ShapeInfo si = shape_info(plan.shape);
  const hipError_t e =
      si.stream ? launch_attn_stream(p, si.local, stream) : launch_attn_mfma(p, si.local, plan.kv_fp8, plan.br_fp8, stream);
  if (e != hipSuccess) return LA_ERR_LAUNCH;
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

}  // extern "C"
