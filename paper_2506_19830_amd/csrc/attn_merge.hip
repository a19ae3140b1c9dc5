// Merge of the split-prefix partials of verify attention (gfx950).
//
// Every (row tile, kv head, chunk) workgroup of the MFMA kernel leaves an
// unnormalised partial (O_s, m_s, l_s) per query row, m in log2 units.  The exact
// softmax over the union of the chunks is
//     M = max_s m_s,   w_s = 2^(m_s - M),   O = sum_s w_s O_s / sum_s w_s l_s,
//     lse = ln2 * (M + log2 sum_s w_s l_s).
// One wavefront owns one output row: lane s < n_s loads (m_s, l_s), the maximum
// and the denominator are wavefront shuffle reductions, the weights are then
// broadcast lane by lane while each lane accumulates its two output columns.
#include "la_internal.hpp"

namespace la {
namespace {

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

constexpr int kD = 128;
constexpr int kWaves = 4;

__global__ __launch_bounds__(64 * kWaves) void attn_merge_kernel(const AttnParams p) {
  const int lane = threadIdx.x & 63;
  const size_t grow = (size_t)blockIdx.x * kWaves + (threadIdx.x >> 6);  // row over all requests
  if (grow >= (size_t)p.B * p.n_rows) return;
  const int b = (int)(grow / p.n_rows);
  const int r = (int)(grow % p.n_rows);
  const int n_s = attn_num_chunks(p.prefix_lens[b], p.chunk_len);
  const size_t slot0 = (size_t)b * p.s_max;

  float acc0 = 0.f, acc1 = 0.f, m_all = -INFINITY, denom = 0.f;
  // more than 64 chunks are folded 64 at a time with the usual running rescale
  for (int s0 = 0; s0 < n_s; s0 += 64) {
    const int cnt = min(64, n_s - s0);
    float m = -INFINITY, l = 0.f;
    if (lane < cnt) {
      const f32x2 ml = *(const f32x2 *)(p.part_ml + ((slot0 + s0 + lane) * p.n_rows + r) * 2);
      m = ml.x;
      l = ml.y;
    }
    float mx = m;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    const float m_new = fmaxf(m_all, mx);
    const float w = (lane < cnt) ? __builtin_amdgcn_exp2f(m - m_new) : 0.f;
    float wl = w * l;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) wl += __shfl_xor(wl, off);
    const float rescale = __builtin_amdgcn_exp2f(m_all - m_new);  // 0 on the first pass (m_all = -inf)
    acc0 *= rescale;
    acc1 *= rescale;
    denom = denom * rescale + wl;
    m_all = m_new;
    const float *po = p.part_o + ((slot0 + s0) * p.n_rows + r) * kD + 2 * lane;
    const size_t stride = (size_t)p.n_rows * kD;  // between the partials of consecutive chunks
    // with many chunks this loop is bound by the latency of its loads, so a whole group of 32 partial rows is
    // requested before the first is used (64 registers)
#pragma unroll 1
    for (int g = 0; g < cnt; g += 32) {
      f32x2 o[32];
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        const int sj = g + j < cnt ? g + j : cnt - 1;   // surplus slots repeat the last chunk with weight zero
        o[j] = *(const f32x2 *)(po + (size_t)sj * stride);
      }
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        const float ws = g + j < cnt ? __shfl(w, g + j) : 0.f;
        acc0 = __builtin_fmaf(ws, o[j].x, acc0);
        acc1 = __builtin_fmaf(ws, o[j].y, acc1);
      }
    }
  }
  const float inv = 1.0f / denom;
  acc0 *= inv;
  acc1 *= inv;
  const size_t orow = grow * kD + 2 * lane;
  if (p.out_f32) {
    f32x2 v = {acc0, acc1};
    *(f32x2 *)((float *)p.out + orow) = v;
  } else {
    f32x2 v = {acc0, acc1};
    *(bf16x2 *)((__bf16 *)p.out + orow) = __builtin_convertvector(v, bf16x2);
  }
  if (p.lse && lane == 0) p.lse[grow] = 0.69314718055994530942f * (m_all + __builtin_log2f(denom));
}

// Few chunks (at most kFew per request), the usual case with many query rows: 32 threads own one row, four output
// columns each.  Every thread forms the weights of its row itself (the (m, l) pairs are one broadcast load each) and
// has all its 16-byte partial loads in flight at once; nothing is exchanged between lanes.
constexpr int kFew = 8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;

__global__ __launch_bounds__(256) void attn_merge_few_kernel(const AttnParams p) {
  const size_t grow = (size_t)blockIdx.x * 8 + (threadIdx.x >> 5);  // row over all requests
  if (grow >= (size_t)p.B * p.n_rows) return;
  const int col = (threadIdx.x & 31) * 4;
  const int b = (int)(grow / p.n_rows);
  const int r = (int)(grow % p.n_rows);
  const int n_s = attn_num_chunks(p.prefix_lens[b], p.chunk_len);  // <= kFew (checked by the host)
  const size_t slot0 = (size_t)b * p.s_max;
  const size_t stride = (size_t)p.n_rows * kD;
  const float *po = p.part_o + (slot0 * p.n_rows + r) * kD + col;
  const float *pml = p.part_ml + (slot0 * p.n_rows + r) * 2;

  f32x4 o[kFew];
  float m[kFew], l[kFew];
#pragma unroll
  for (int s = 0; s < kFew; ++s) {
    const int sc = s < n_s ? s : n_s - 1;  // surplus slots repeat the last chunk with weight zero
    o[s] = *(const f32x4 *)(po + (size_t)sc * stride);
    const f32x2 ml = *(const f32x2 *)(pml + (size_t)sc * p.n_rows * 2);
    m[s] = s < n_s ? ml.x : -INFINITY;
    l[s] = ml.y;
  }
  float m_all = m[0];
#pragma unroll
  for (int s = 1; s < kFew; ++s) m_all = fmaxf(m_all, m[s]);
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  float denom = 0.f;
#pragma unroll
  for (int s = 0; s < kFew; ++s) {
    const float w = __builtin_amdgcn_exp2f(m[s] - m_all);  // 0 for surplus slots
    denom = __builtin_fmaf(w, l[s], denom);
    acc += o[s] * w;
  }
  const float inv = 1.0f / denom;
  acc *= inv;
  const size_t orow = grow * kD + col;
  if (p.out_f32)
    *(f32x4 *)((float *)p.out + orow) = acc;
  else
    *(bf16x4 *)((__bf16 *)p.out + orow) = __builtin_convertvector(acc, bf16x4);
  if (p.lse && col == 0) p.lse[grow] = 0.69314718055994530942f * (m_all + __builtin_log2f(denom));
}

}  // namespace

hipError_t launch_attn_merge(const AttnParams &p, hipStream_t stream) {
  ProfileScope scope(SLOT_ATTN_MERGE, stream);
  const size_t rows = (size_t)p.B * p.n_rows;
  if (p.s_max <= kFew) {
    hipLaunchKernelGGL(attn_merge_few_kernel, dim3((unsigned)((rows + 7) / 8)), dim3(256), 0, stream, p);
    return hipGetLastError();
  }
  const int grid = (int)((rows + kWaves - 1) / kWaves);
  hipLaunchKernelGGL(attn_merge_kernel, dim3(grid), dim3(64 * kWaves), 0, stream, p);
  return hipGetLastError();
}

}  // namespace la
