// Verify attention for fp32 tensors (gfx950), the small-case / reference-precision path.
//
// One wavefront owns one query row (request b, branch g, token i, head h) and walks
// its visible keys -- the request's prefix through the block table, then the part of
// the request's drafted chain its branch sees, then tokens 0..i of its own branch
// (Algorithm 1: a branch sees the shared prefix, the drafted steps before it and only
// its own continuation) -- 64 at a time:
//   lane k   : score of key k0+k (full dot product over D, fp32 FMA chain)
//   wavefront: running max / sum by shuffle reductions (online softmax)
//   lane d   : output columns d, d+64, ... accumulate p_k * V[k][d], p_k broadcast by shuffle
// No workspace, no split: the sizes this path serves are tiny.
#include "la_internal.hpp"

namespace la {
namespace {

constexpr int kWaves = 4;

template <int D>
__global__ __launch_bounds__(64 * kWaves) void attn_f32_kernel(const AttnParams p) {
  __shared__ float q_lds[kWaves][D];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t total_rows = (size_t)p.B * p.n_rows;
  const size_t want = (size_t)blockIdx.x * kWaves + wave;
  const bool valid = want < total_rows;
  const size_t grow = valid ? want : total_rows - 1;  // surplus wavefronts redo the last row and store nothing
  const int b = (int)(grow / p.n_rows);
  const int r = (int)(grow % p.n_rows);
  const int h = r % p.Hq, t = r / p.Hq;  // t = g*L + i
  const int i = t % p.L, bstart = t - i;
  const int kvh = h / p.G;
  const int P = p.prefix_lens[b];
  // nested form: the first `vis` chain tokens are keys.  Tree form: all C pool tokens are walked and the ones
  // whose segment the branch does not see score -inf.
  const bool tree = p.pool_seg != nullptr;
  const int vis = p.C > 0 ? (tree ? p.C : p.chain_vis[b * p.gamma + t / p.L]) : 0;
  const uint64_t seen = tree ? p.seg_mask[b * p.gamma + t / p.L] : 0;
  const int n_keys = P + vis + i + 1;

  const float *q = (const float *)p.q + grow * D;
  for (int d = lane; d < D; d += 64) q_lds[wave][d] = q[d];
  __syncthreads();

  const float *kc = (const float *)p.k_cache, *vc = (const float *)p.v_cache;
  const float *kb = (const float *)p.k_branch + ((size_t)b * p.gamma * p.L * p.Hkv + kvh) * D;
  const float *vb = (const float *)p.v_branch + ((size_t)b * p.gamma * p.L * p.Hkv + kvh) * D;
  const float *kn = (const float *)p.k_chain + ((size_t)b * p.C * p.Hkv + kvh) * D;
  const float *vn = (const float *)p.v_chain + ((size_t)b * p.C * p.Hkv + kvh) * D;
  const int32_t *table = p.block_tables ? p.block_tables + (size_t)b * p.max_blocks : nullptr;

  // row of key `key` in the K tensors (k = true) or the V tensors
  auto kv_row = [&](int key, bool k) -> const float * {
    if (key < P) {
      const int lb = key / p.block_size;
      const int blk = table ? table[lb] : b * p.max_blocks + lb;
      return (k ? kc : vc) + (((size_t)blk * p.Hkv + kvh) * p.block_size + key % p.block_size) * D;
    }
    if (key < P + vis) return (k ? kn : vn) + (size_t)(key - P) * p.Hkv * D;
    return (k ? kb : vb) + (size_t)(bstart + key - P - vis) * p.Hkv * D;
  };

  constexpr int E = D / 64;
  float acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  for (int k0 = 0; k0 < n_keys; k0 += 64) {
    const int key = k0 + lane;
    float s = -INFINITY;
    if (key < n_keys) {
      const float *krow = kv_row(key, true);
      float dot = 0.f;
#pragma unroll 8
      for (int d = 0; d < D; ++d) dot = __builtin_fmaf(q_lds[wave][d], krow[d], dot);
      s = dot * p.scale_log2;
      if (tree && key >= P && key < P + vis && !((seen >> p.pool_seg[(size_t)b * p.C + (key - P)]) & 1)) s = -INFINITY;
    }
    float mx = s;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    // finite unless nothing has been visible so far (tree form: a group of unseen pool tokens and no prefix)
    const float m_new = fmaxf(m_run, mx);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float pr = __builtin_amdgcn_exp2f(s - m_use);
    float sum = pr;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
    l_run = l_run * alpha + sum;
    m_run = m_new;
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] *= alpha;
    const int cnt = min(64, n_keys - k0);
    for (int j = 0; j < cnt; ++j) {
      const float pj = __shfl(pr, j);
      const float *vrow = kv_row(k0 + j, false);
#pragma unroll
      for (int e = 0; e < E; ++e) acc[e] = __builtin_fmaf(pj, vrow[lane + 64 * e], acc[e]);
    }
  }
  if (!valid) return;
  const float inv = 1.0f / l_run;
  float *out = (float *)p.out + grow * D;
#pragma unroll
  for (int e = 0; e < E; ++e) out[lane + 64 * e] = acc[e] * inv;
  if (p.lse && lane == 0) p.lse[grow] = 0.69314718055994530942f * (m_run + __builtin_log2f(l_run));
}

}  // namespace

hipError_t launch_attn_f32(const AttnParams &p, hipStream_t stream) {
  ProfileScope scope(SLOT_ATTN_F32, stream);
  const size_t rows = (size_t)p.B * p.n_rows;
  const int grid = (int)((rows + kWaves - 1) / kWaves);
  switch (p.D) {
    case 64:
      hipLaunchKernelGGL(attn_f32_kernel<64>, dim3(grid), dim3(64 * kWaves), 0, stream, p);
      break;
    case 128:
      hipLaunchKernelGGL(attn_f32_kernel<128>, dim3(grid), dim3(64 * kWaves), 0, stream, p);
      break;
    case 256:
      hipLaunchKernelGGL(attn_f32_kernel<256>, dim3(grid), dim3(64 * kWaves), 0, stream, p);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace la
