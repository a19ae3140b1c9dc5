// Internal declarations shared by the host API and the kernel translation units
// of libla_verify (gfx950 only).  Nothing here is part of the public C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "la_verify.h"

namespace la {

// ----------------------------------------------------------------------------
// Verify attention.
//
// Rows that share one KV head: r = (g*L + i)*G + hh  for branch g, token i and
// query head hh of the group (G = Hq/Hkv); R = gamma*L*G of them per request.
// The prefix of request b is cut into n_chunks(b) = max(1, ceil(P_b/chunk_len))
// chunks; one workgroup reduces (row tile, kv head, chunk) and the one that owns
// the last chunk also reduces the branch-private keys.  Each writes an
// unnormalised partial (O, m, l) that the merge kernel combines.
// ----------------------------------------------------------------------------
struct AttnParams {
  const void *q, *k_cache, *v_cache, *k_branch, *v_branch;
  // nested branches: a chain of C drafted tokens per request [B, C, Hkv, D] (branch storage type); branch g of
  // request b sees chain tokens 0 .. chain_vis[b*gamma + g] - 1, between the prefix and its own tokens.  C == 0: none
  const void *k_chain, *v_chain;
  const int32_t *chain_vis;
  int C;
  // tree form (pool_seg != nullptr): the C tokens are a pool; token c of request b belongs to segment
  // pool_seg[b*C + c] (0..63) and branch g sees the tokens whose segment bit is set in seg_mask[b*gamma + g]
  const int32_t *pool_seg;
  const uint64_t *seg_mask;
  const int32_t *block_tables, *prefix_lens;
  const float *k_scale, *v_scale;
  float *part_o;   // [B, s_max, n_rows, D]
  float *part_ml;  // [B, s_max, n_rows, 2]  (running max in log2 units, sum)
  void *out;       // [B, n_rows, D]
  float *lse;      // [B, n_rows] or null
  int B, Hq, Hkv, G, D, gamma, L;
  int block_size, block_shift, max_blocks;  // block_size = 1 << block_shift
  int R;            // gamma*L*G
  int n_rows;       // gamma*L*Hq
  int n_row_tiles;  // ceil(R / tile_m)
  int chunk_len;    // nominal prefix tokens per chunk, multiple of 64 (see attn_chunk_range)
  int last_short;   // tiles of other work the last chunk is counted as carrying
  int s_max;        // partial slots per request = max_b n_chunks(b)
  int total_units;  // sum_b n_chunks(b)
  int out_f32;      // output dtype: 1 = fp32, 0 = bf16
  int q_type, kv_type, br_type;  // la_dtype of Q, of the prefix cache, of the branch / chain / pool K and V
  float scale_log2; // softmax_scale * log2(e)
  int force_again;  // streaming shapes (fp8): start with the give-up flag raised, so that every workgroup also runs its
                    // second attempt (a self-test hook of the benchmark library; 0 otherwise)
  // With few requests what a workgroup needs to find its chunk travels in the kernel arguments, prepared by the host
  // from its copy of the prefix lengths, so that no kernel start waits on a dependent load of prefix_lens or on
  // integer divisions: n_inline = B if B <= kMaxInlineLens, else 0.
  int n_inline;
  struct Req {
    int P;          // prefix length
    int n;          // chunks
    int q, r;       // (tiles + last_short) = q*n + r
    uint32_t inv;   // floor(2^32 / n) + 1: floor(x / n) == (x * inv) >> 32 for x < 2^32 / n
  } req[8];
};
constexpr int kMaxInlineLens = 8;

__host__ __device__ inline int attn_num_chunks(int prefix_len, int chunk_len) {
  int n = (prefix_len + chunk_len - 1) / chunk_len;
  return n < 1 ? 1 : n;
}

// Token range [*k_begin, *k_end) of chunk c of a prefix of P tokens.  chunk_len only fixes the number of chunks
// n = attn_num_chunks(P, chunk_len); the T = ceil(P/64) key tiles are then dealt out evenly (sizes differ by at most
// one tile), with the last chunk, whose workgroup also reduces the branch-private keys, counted as carrying
// `last_short` tiles of other work.  A chunk may come out empty (k_begin == k_end) when n is close to T.
__host__ __device__ inline void attn_chunk_range(int P, int chunk_len, int last_short, int c, int *k_begin,
                                                 int *k_end) {
  const long long n = attn_num_chunks(P, chunk_len);
  const long long T = ((long long)P + 63) / 64;
  const long long Tv = T + last_short;
  long long t0 = c * Tv / n, t1 = (c + 1) * Tv / n;
  if (t0 > T) t0 = T;
  if (t1 > T || c == n - 1) t1 = T;
  const long long e = t1 * 64 < P ? t1 * 64 : P;
  *k_begin = (int)(t0 * 64);
  *k_end = (int)e;
}
// upper bound of a chunk's length in tokens under attn_chunk_range
__host__ __device__ inline int attn_max_chunk_tokens(int chunk_len, int last_short) {
  return chunk_len + 64 * (last_short + 2);
}

enum KernelSlot {
  SLOT_ATTN_MFMA = 0,
  SLOT_ATTN_MERGE,
  SLOT_ATTN_F32,
  SLOT_ACCEPT_STATS,
  SLOT_ACCEPT_WARP,
  SLOT_ACCEPT_DECIDE,
  SLOT_ACCEPT_RESID,
  SLOT_ACCEPT_PICK,
  SLOT_KV_COMMIT,
  SLOT_CALIB_MFMA,
  SLOT_CALIB_READ,
  SLOT_COUNT
};

// The MFMA kernel is built in a few (wavefronts, row blocks per wavefront) shapes.
int attn_mfma_num_shapes();
int attn_mfma_tile_m(int shape);   // rows per workgroup of a shape
int attn_mfma_wgs_per_cu(int shape);  // workgroups of a shape that fit on one CU (LDS)
int attn_mfma_max_chunk_blocks();  // a chunk may span at most this many cache blocks
hipError_t launch_attn_mfma(const AttnParams &p, int shape, bool kv_fp8, bool br_fp8, hipStream_t stream);
// The streaming shapes (few rows per KV head; fp8 cache and fp8 branch K/V, flat calls): row blocks x key slices.
int attn_stream_num_shapes();
int attn_stream_tile_m(int shape);
int attn_stream_step_keys(int shape);  // keys a workgroup advances per pipeline step
int attn_stream_max_chunk_blocks();
bool attn_stream_shape_is_fp8(int shape);  // else: bf16 cache and branch K/V
hipError_t launch_attn_stream(const AttnParams &p, int shape, hipStream_t stream);
hipError_t launch_attn_merge(const AttnParams &p, hipStream_t stream);
hipError_t launch_attn_f32(const AttnParams &p, hipStream_t stream);

// ----------------------------------------------------------------------------
// Speculative accept / resample.
// ----------------------------------------------------------------------------
struct AcceptParams {
  const void *target, *draft;  // [NB, K+1, V], [NB, K, V]
  const int32_t *tokens;       // [NB, K]
  const float *u_accept, *u_sample;
  int32_t *accepted_len, *next_token;
  float *ratio;                // [NB, K] or null
  int NB, K, V, bf16;
  int n_chunks;                // slices of the fp32 statistics pass per row
  int n_fine;                  // 2048-token slices of the fp64 resampling path per row
  float inv_temp_log2;         // log2(e) / T
  double inv_temp;             // 1 / T
  // workspace
  float *stats;                // [rows = NB*(2K+1), n_chunks, 2]  (exact max, sum 2^((x-max)*log2e/T))
  int32_t *n_acc;              // [NB]
  double *zsum;                // [NB, 2, n_fine]  fp64 sum exp(z - max) of the resampling rows
  double *rsum;                // [NB, 2, n_fine]  fp64 slice sums of the residual and of p
  float *rowmax;               // [NB, 2] exact row maxima (raw logits) of the resampling rows
  double *lane_sums;           // [NB, n_fine, 256, 2] per-lane sums of the residual and of p
  // top-k / top-p warping of the target rows (off: top_k == 0 and top_p >= 1)
  int top_k;
  float top_p;
  uint32_t *warp_key;          // [NB*(K+1)] order-preserving key of the smallest logit a row keeps
  double *warp_z;              // [NB*(K+1)] sum exp((x - max)/T) over the kept tokens
  float *warp_max;             // [NB*(K+1)] row maximum (raw logits)
  double *warp_zs;             // [NB*(K+1), n_fine] fp64 slice sums of exp((x - max)/T) of every target row (top-p alone)
};

size_t accept_workspace_bytes(int NB, int K, int V, bool bf16, int *n_chunks_out, int *n_fine_out);
void accept_carve_workspace(AcceptParams &p, void *ws);
hipError_t launch_accept(const AcceptParams &p, hipStream_t stream);
// out[i] = the accept path's own fp64 exponential of y[i] (self-test hook)
hipError_t launch_exp64_probe(const double *y, double *out, size_t n, hipStream_t stream);

// ----------------------------------------------------------------------------
// KV commit.
// ----------------------------------------------------------------------------
struct CommitParams {
  void *k_cache, *v_cache;  // [layers][num_blocks, Hkv, block_size, D], written
  const void *k_branch, *v_branch, *k_chain, *v_chain;
  const int32_t *block_tables, *prefix_lens, *src_branch, *n_chain, *n_own;
  const float *k_scale, *v_scale;
  // tree form: k_chain / v_chain are the pool, pool_seg [B, C] the node of each pool token, commit_mask [B] the
  // accepted nodes; n_chain is unused.  pool_seg == nullptr selects the chain form.
  const int32_t *pool_seg;
  const uint64_t *commit_mask;
  int32_t *new_prefix_lens;
  int B, Hkv, D, gamma, L, C, block_size, block_shift, max_blocks, num_layers;
  int capacity;                                                     // max_blocks * block_size
  int64_t cache_stride, branch_stride, chain_stride, scale_stride;  // elements between consecutive layers
};
// src_bytes: storage size of a source element; quantise: bf16 source into an fp8 cache
hipError_t launch_kv_commit(const CommitParams &p, int src_bytes, bool quantise, hipStream_t stream);

// ----------------------------------------------------------------------------
// Optional per-kernel event timing.  The two hooks are defined only in the benchmark build of the library
// (bench_aids.hip, see la_verify_bench.h); in the product library they are absent, the references below resolve
// to null and a launch does nothing beside launching.
// ----------------------------------------------------------------------------
__attribute__((weak)) void *profile_before(int slot, hipStream_t stream);            // start event, or null
__attribute__((weak)) void profile_after(int slot, hipStream_t stream, void *start);
// self-test hook of the benchmark library: nonzero = the fp8 streaming kernels run their second attempt everywhere
__attribute__((weak)) int selftest_force_second_attempt();

struct ProfileScope {
  int slot;
  hipStream_t stream;
  void *start;
  ProfileScope(int s, hipStream_t st) : slot(s), stream(st), start(profile_before ? profile_before(s, st) : nullptr) {}
  ~ProfileScope() {
    if (start && profile_after) profile_after(slot, stream, start);
  }
};

}  // namespace la
