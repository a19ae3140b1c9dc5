// Verify attention, the general path (gfx950): fp32 tensors (the small-case / reference-precision configuration), and
// bf16 / fp8-e4m3 storage at the head dimensions the MFMA kernels are not written for (64 and 256).  All arithmetic is
// fp32 on exactly widened inputs.
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

// element i of a tensor stored as T, widened to fp32 (exact)
template <int T>
__device__ __forceinline__ float load_elem(const void *base, size_t i) {
  if constexpr (T == LA_F32) {
    return ((const float *)base)[i];
  } else if constexpr (T == LA_BF16) {
    const uint32_t w = (uint32_t)((const uint16_t *)base)[i] << 16;
    return __builtin_bit_cast(float, w);
  } else {
    const auto v = __builtin_amdgcn_cvt_pk_f32_fp8((int)((const uint8_t *)base)[i], false);
    return v[0];
  }
}
__device__ __forceinline__ float load_elem_rt(int type, const void *base, size_t i) {
  return type == LA_F32 ? load_elem<LA_F32>(base, i) : load_elem<LA_BF16>(base, i);
}

// D: head dimension; KV, BR: storage type of the prefix cache and of the branch / chain / pool K and V (compile time:
// they sit in the inner loops); Q and output types are read from the parameters.
template <int D, int KV, int BR>
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

  for (int d = lane; d < D; d += 64) q_lds[wave][d] = load_elem_rt(p.q_type, p.q, grow * D + d);
  __syncthreads();

  // an fp8 tensor is stored divided by its head's scale: K's scale multiplies the score, V's the weighted value
  float ks_pre = 1.f, vs_pre = 1.f, ks_br = 1.f, vs_br = 1.f;
  if (KV == LA_FP8_E4M3) ks_pre = p.k_scale ? p.k_scale[kvh] : 1.f, vs_pre = p.v_scale ? p.v_scale[kvh] : 1.f;
  if (BR == LA_FP8_E4M3) ks_br = ks_pre, vs_br = vs_pre;
  const int32_t *table = p.block_tables ? p.block_tables + (size_t)b * p.max_blocks : nullptr;

  // element d of the row of key `key` in the K tensors (k = true) or the V tensors; the row's element index first
  auto kv_index = [&](int key, int &seg) -> size_t {
    if (key < P) {
      const int lb = key / p.block_size;
      const int blk = table ? table[lb] : b * p.max_blocks + lb;
      seg = 0;
      return (((size_t)blk * p.Hkv + kvh) * p.block_size + key % p.block_size) * D;
    }
    if (key < P + vis) {
      seg = 1;
      return (((size_t)b * p.C + (key - P)) * p.Hkv + kvh) * D;
    }
    seg = 2;
    return (((size_t)b * p.gamma * p.L + bstart + key - P - vis) * p.Hkv + kvh) * D;
  };
  auto kv_elem = [&](bool k, int seg, size_t idx) -> float {
    if (seg == 0) return load_elem<KV>(k ? p.k_cache : p.v_cache, idx);
    if (seg == 1) return load_elem<BR>(k ? p.k_chain : p.v_chain, idx);
    return load_elem<BR>(k ? p.k_branch : p.v_branch, idx);
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
      int seg;
      const size_t krow = kv_index(key, seg);
      float dot = 0.f;
#pragma unroll 8
      for (int d = 0; d < D; ++d) dot = __builtin_fmaf(q_lds[wave][d], kv_elem(true, seg, krow + d), dot);
      s = dot * p.scale_log2 * (seg == 0 ? ks_pre : ks_br);
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
      int seg;
      const size_t vrow = kv_index(k0 + j, seg);
      const float pj = __shfl(pr, j) * (seg == 0 ? vs_pre : vs_br);
#pragma unroll
      for (int e = 0; e < E; ++e) acc[e] = __builtin_fmaf(pj, kv_elem(false, seg, vrow + lane + 64 * e), acc[e]);
    }
  }
  if (!valid) return;
  const float inv = 1.0f / l_run;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const float o = acc[e] * inv;
    if (p.out_f32) {
      ((float *)p.out)[grow * D + lane + 64 * e] = o;
    } else {  // bf16, round to nearest even
      const uint32_t u = __builtin_bit_cast(uint32_t, o);
      ((uint16_t *)p.out)[grow * D + lane + 64 * e] = (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
    }
  }
  if (p.lse && lane == 0) p.lse[grow] = 0.69314718055994530942f * (m_run + __builtin_log2f(l_run));
}

template <int KV, int BR>
hipError_t launch_typed(const AttnParams &p, hipStream_t stream) {
  const size_t rows = (size_t)p.B * p.n_rows;
  const int grid = (int)((rows + kWaves - 1) / kWaves);
  switch (p.D) {
    case 64:
      hipLaunchKernelGGL((attn_f32_kernel<64, KV, BR>), dim3(grid), dim3(64 * kWaves), 0, stream, p);
      break;
    case 128:
      hipLaunchKernelGGL((attn_f32_kernel<128, KV, BR>), dim3(grid), dim3(64 * kWaves), 0, stream, p);
      break;
    case 256:
      hipLaunchKernelGGL((attn_f32_kernel<256, KV, BR>), dim3(grid), dim3(64 * kWaves), 0, stream, p);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_f32(const AttnParams &p, hipStream_t stream) {
  ProfileScope scope(SLOT_ATTN_F32, stream);
  if (p.kv_type == LA_F32 && p.br_type == LA_F32) return launch_typed<LA_F32, LA_F32>(p, stream);
  if (p.kv_type == LA_BF16 && p.br_type == LA_BF16) return launch_typed<LA_BF16, LA_BF16>(p, stream);
  if (p.kv_type == LA_FP8_E4M3 && p.br_type == LA_FP8_E4M3) return launch_typed<LA_FP8_E4M3, LA_FP8_E4M3>(p, stream);
  if (p.kv_type == LA_FP8_E4M3 && p.br_type == LA_BF16) return launch_typed<LA_FP8_E4M3, LA_BF16>(p, stream);
  return hipErrorInvalidValue;
}

}  // namespace la
