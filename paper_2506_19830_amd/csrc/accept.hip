// Token-level speculative accept / resample over the vocabulary (gfx950).
//
// Section 2 ("Speculative Decoding"): the K drafted tokens of a branch are examined in
// order, x_i accepted with probability min(1, p_i(x_i)/q_i(x_i)); the first rejection n
// stops the walk and one token is drawn from norm(max(0, p_n - q_n)); with all K accepted
// a bonus token is drawn from p_K.
//
// Four launches:
//   stats   one coalesced pass over every logit row (NB*(2K+1) rows x V): per
//           (row, vocabulary slice) the exact maximum and sum 2^((x-max)*log2e/T), fp32.
//           This is the HBM-bound part: each logit is read exactly once.
//   decide  per branch: fold the slice statistics, gather p_i(x_i), q_i(x_i), test
//           u*q < p in order, write n.  Also starts the fp64 resampling path:
//   resid   (two phases in one kernel file) fp64 normaliser of the two rows at position n,
//           then fp64 slice sums of max(0, p-q) (and of p, the fallback when the residual
//           has no mass, and the distribution of the bonus token).
//   pick    per branch: locate the slice in which the running sum first exceeds
//           u_sample * total, then the token inside it (block scan in token order).
// The resampling rows are re-read (2 rows of NB*(2K+1)); they are L2/Infinity-Cache hits.
// fp64 there makes the blocked running sum agree with a sequential one to ~1e-16, so the
// drawn token does not depend on the summation order.
#include <limits.h>

#include "la_internal.hpp"

namespace la {
namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kThreads = 256;
constexpr int kPer = 32;                    // elements per thread per slice
constexpr int kChunk = kThreads * kPer;     // 8192 vocabulary entries per slice

// (bit-casting a vector element in place, __builtin_bit_cast(float, w[k]), reads element 0 with this compiler;
// pass the element by value instead)
__device__ __forceinline__ float as_f32(uint32_t w) { return __builtin_bit_cast(float, w); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xFFFF0000u); }

__device__ __forceinline__ float load_logit(const void *base, size_t idx, bool bf16) {
  if (bf16) return __builtin_bit_cast(float, (uint32_t)((const uint16_t *)base)[idx] << 16);
  return ((const float *)base)[idx];
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// row rw of the stacked [target rows ; draft rows] list
__device__ __forceinline__ const uint8_t *stacked_row(const AcceptParams &p, int rw) {
  const size_t esz = p.bf16 ? 2 : 4;
  const int n_t = p.NB * (p.K + 1);
  if (rw < n_t) return (const uint8_t *)p.target + (size_t)rw * p.V * esz;
  return (const uint8_t *)p.draft + (size_t)(rw - n_t) * p.V * esz;
}

// ---------------------------------------------------------------------------------------------
// stats: grid (n_chunks, rows)
// ---------------------------------------------------------------------------------------------
template <bool BF16, bool VEC>
__global__ __launch_bounds__(kThreads) void accept_stats_kernel(const AcceptParams p) {
  __shared__ float red[2][kThreads / 64];
  const int c = blockIdx.x, rw = blockIdx.y;
  const int tid = threadIdx.x;
  const uint8_t *row = stacked_row(p, rw);
  const int v0 = c * p.chunk;
  const int v1 = min(p.V, v0 + p.chunk);

  float x[kPer];
  if constexpr (VEC) {
    constexpr int per_vec = BF16 ? 8 : 4;           // elements per 16-byte load
    constexpr int n_vec = kPer / per_vec;           // loads per thread
#pragma unroll
    for (int e = 0; e < n_vec; ++e) {
      const int v = v0 + (e * kThreads + tid) * per_vec;   // consecutive lanes read consecutive 16 B
      u32x4 w = {0, 0, 0, 0};
      const bool in = v < v1;                       // V % per_vec == 0 on this path, so a vector is all-in or all-out
      if (in) w = *(const u32x4 *)(row + (size_t)v * (BF16 ? 2 : 4));
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if constexpr (BF16) {
          x[e * 8 + 2 * k] = in ? bf16_lo(w[k]) : -INFINITY;
          x[e * 8 + 2 * k + 1] = in ? bf16_hi(w[k]) : -INFINITY;
        } else {
          x[e * 4 + k] = in ? as_f32(w[k]) : -INFINITY;
        }
      }
    }
  } else {
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      const int v = v0 + e * kThreads + tid;
      x[e] = v < v1 ? load_logit(row, v, BF16) : -INFINITY;
    }
  }
  float m = -INFINITY;
#pragma unroll
  for (int e = 0; e < kPer; ++e) m = fmaxf(m, x[e]);
  m = wave_max(m);
  if ((tid & 63) == 0) red[0][tid >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));   // slice maximum (finite: slice not empty)
  const float cm = -m * p.inv_temp_log2;
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < kPer; ++e) s += __builtin_amdgcn_exp2f(__builtin_fmaf(x[e], p.inv_temp_log2, cm));
  s = wave_sum(s);
  if ((tid & 63) == 0) red[1][tid >> 6] = s;
  __syncthreads();
  if (tid == 0) {
    f32x2 out = {m, (red[1][0] + red[1][1]) + (red[1][2] + red[1][3])};
    *(f32x2 *)(p.stats + ((size_t)rw * p.n_chunks + c) * 2) = out;
  }
}

// fold the slice statistics of one row: maximum and sum 2^((x-max)*c)
__device__ __forceinline__ void fold_row(const AcceptParams &p, int rw, float &m_out, float &z_out) {
  const float *st = p.stats + (size_t)rw * p.n_chunks * 2;
  float m = -INFINITY;
  for (int c = 0; c < p.n_chunks; ++c) m = fmaxf(m, st[2 * c]);
  float z = 0.f;
  for (int c = 0; c < p.n_chunks; ++c) z += st[2 * c + 1] * __builtin_amdgcn_exp2f((st[2 * c] - m) * p.inv_temp_log2);
  m_out = m;
  z_out = z;
}

// ---------------------------------------------------------------------------------------------
// decide: grid NB, one wavefront; lane i handles drafted position i (looping when K > 64)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void accept_decide_kernel(const AcceptParams p) {
  const int nb = blockIdx.x, lane = threadIdx.x;
  const int n_t = p.NB * (p.K + 1);
  int first_reject = p.K;
  for (int i0 = 0; i0 < p.K; i0 += 64) {
    const int i = i0 + lane;
    bool reject = false;
    if (i < p.K) {
      const int rt = nb * (p.K + 1) + i, rd = n_t + nb * p.K + i;
      float mp, zp, mq, zq;
      fold_row(p, rt, mp, zp);
      fold_row(p, rd, mq, zq);
      const int x = p.tokens[(size_t)nb * p.K + i];
      const float tx = load_logit(p.target, (size_t)rt * p.V + x, p.bf16);
      const float dx = load_logit(p.draft, (size_t)(rd - n_t) * p.V + x, p.bf16);
      const float px = __builtin_amdgcn_exp2f((tx - mp) * p.inv_temp_log2) / zp;
      const float qx = __builtin_amdgcn_exp2f((dx - mq) * p.inv_temp_log2) / zq;
      const float u = p.u_accept[(size_t)nb * p.K + i];
      reject = !(u * qx < px);
      if (p.ratio) p.ratio[(size_t)nb * p.K + i] = px / qx;
    }
    const unsigned long long mask = __ballot(reject);
    if (mask && first_reject == p.K) first_reject = i0 + __builtin_ctzll(mask);
  }
  if (lane == 0) {
    const int n = first_reject;
    p.accepted_len[nb] = n;
    p.n_acc[nb] = n;
    // exact maxima of the resampling rows: target row n, draft row n (unused when n == K)
    float m, z;
    fold_row(p, nb * (p.K + 1) + n, m, z);
    p.rowmax[2 * nb] = m;
    if (n < p.K) {
      fold_row(p, n_t + nb * p.K + n, m, z);
      p.rowmax[2 * nb + 1] = m;
    } else {
      p.rowmax[2 * nb + 1] = 0.f;
    }
  }
}

// fp64 probability mass (unnormalised) of one logit: exp(x/T - max/T)
__device__ __forceinline__ double mass64(float x, double mx_over_t, double temperature) {
  return exp((double)x / temperature - mx_over_t);
}

// ---------------------------------------------------------------------------------------------
// zsum: grid (n_chunks, NB, 2): fp64 sum exp(z - max) of one slice of a resampling row
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void accept_zsum_kernel(const AcceptParams p) {
  __shared__ double red[kThreads / 64];
  const int c = blockIdx.x, nb = blockIdx.y, which = blockIdx.z;
  const int tid = threadIdx.x;
  const int n = p.n_acc[nb];
  double total = 0.0;
  if (!(which == 1 && n == p.K)) {
    const size_t rowi = which == 0 ? (size_t)nb * (p.K + 1) + n : (size_t)nb * p.K + n;
    const void *base = which == 0 ? p.target : p.draft;
    const double mt = (double)p.rowmax[2 * nb + which] / p.temperature;
    const int v0 = c * p.chunk, v1 = min(p.V, v0 + p.chunk);
    double s = 0.0;
    // thread t owns the kPer consecutive tokens v0 + t*kPer ..: the same partition as the pick kernel
    for (int e = 0; e < kPer; ++e) {
      const int v = v0 + tid * kPer + e;
      if (v < v1) s += mass64(load_logit(base, rowi * p.V + v, p.bf16), mt, p.temperature);
    }
    s = wave_sum(s);
    if ((tid & 63) == 0) red[tid >> 6] = s;
    __syncthreads();
    total = (red[0] + red[1]) + (red[2] + red[3]);
  }
  if (tid == 0) p.zsum[((size_t)nb * 2 + which) * p.n_chunks + c] = total;
}

__device__ __forceinline__ double fold64(const double *v, int n) {
  double s = 0.0;
  for (int c = 0; c < n; ++c) s += v[c];
  return s;
}

// residual mass and target mass of token v of branch nb (position n), fp64
struct ResidCtx {
  const void *target, *draft;
  size_t trow, drow;
  double mt, mq, zt, zq, temperature;
  bool has_draft, bf16;
  __device__ __forceinline__ void eval(int v, double &r, double &pm) const {
    pm = mass64(load_logit(target, trow + v, bf16), mt, temperature) / zt;
    r = pm;
    if (has_draft) {
      const double qm = mass64(load_logit(draft, drow + v, bf16), mq, temperature) / zq;
      r = pm - qm;
      if (r < 0.0) r = 0.0;
    }
  }
};

__device__ __forceinline__ ResidCtx make_ctx(const AcceptParams &p, int nb) {
  ResidCtx x;
  const int n = p.n_acc[nb];
  x.target = p.target;
  x.draft = p.draft;
  x.trow = ((size_t)nb * (p.K + 1) + n) * p.V;
  x.has_draft = n < p.K;
  x.drow = x.has_draft ? ((size_t)nb * p.K + n) * p.V : 0;
  x.temperature = p.temperature;
  x.mt = (double)p.rowmax[2 * nb] / p.temperature;
  x.mq = (double)p.rowmax[2 * nb + 1] / p.temperature;
  x.zt = fold64(p.zsum + ((size_t)nb * 2 + 0) * p.n_chunks, p.n_chunks);
  x.zq = x.has_draft ? fold64(p.zsum + ((size_t)nb * 2 + 1) * p.n_chunks, p.n_chunks) : 1.0;
  x.bf16 = p.bf16 != 0;
  return x;
}

// ---------------------------------------------------------------------------------------------
// resid: grid (n_chunks, NB): fp64 slice sums of the residual and of p
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void accept_resid_kernel(const AcceptParams p) {
  __shared__ double red[2][kThreads / 64];
  const int c = blockIdx.x, nb = blockIdx.y, tid = threadIdx.x;
  const ResidCtx ctx = make_ctx(p, nb);
  const int v0 = c * p.chunk, v1 = min(p.V, v0 + p.chunk);
  double sr = 0.0, sp = 0.0;
  for (int e = 0; e < kPer; ++e) {
    const int v = v0 + tid * kPer + e;
    if (v < v1) {
      double r, pm;
      ctx.eval(v, r, pm);
      sr += r;
      sp += pm;
    }
  }
  sr = wave_sum(sr);
  sp = wave_sum(sp);
  if ((tid & 63) == 0) red[0][tid >> 6] = sr, red[1][tid >> 6] = sp;
  __syncthreads();
  if (tid == 0) {
    p.rsum[((size_t)nb * 2 + 0) * p.n_chunks + c] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
    p.rsum[((size_t)nb * 2 + 1) * p.n_chunks + c] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
  }
}

// ---------------------------------------------------------------------------------------------
// pick: grid NB
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void accept_pick_kernel(const AcceptParams p) {
  __shared__ double scan[kThreads];
  __shared__ int best;
  __shared__ int last_mass;
  const int nb = blockIdx.x, tid = threadIdx.x;
  const ResidCtx ctx = make_ctx(p, nb);
  const double *rs = p.rsum + ((size_t)nb * 2 + 0) * p.n_chunks;
  double S = fold64(rs, p.n_chunks);
  bool use_p = false;
  if (!(S > 0.0)) {  // the residual has no mass (only through rounding): draw from p_n itself
    rs = p.rsum + ((size_t)nb * 2 + 1) * p.n_chunks;
    S = fold64(rs, p.n_chunks);
    use_p = true;
  }
  const double thr = (double)p.u_sample[nb] * S;
  // slice in which the running sum first exceeds thr
  int cs = p.n_chunks - 1;
  double before = 0.0;
  {
    double acc = 0.0;
    for (int c = 0; c < p.n_chunks; ++c) {
      if (acc + rs[c] > thr) {
        cs = c;
        before = acc;
        break;
      }
      acc += rs[c];
      if (c == p.n_chunks - 1) before = acc - rs[c];
    }
  }
  const int v0 = cs * p.chunk, v1 = min(p.V, v0 + p.chunk);
  double mass[kPer];
  double local = 0.0;
  int my_last = -1;
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    const int v = v0 + tid * kPer + e;
    double r = 0.0, pm = 0.0;
    if (v < v1) ctx.eval(v, r, pm);
    mass[e] = use_p ? pm : r;
    local += mass[e];
    if (mass[e] > 0.0) my_last = v;
  }
  if (tid == 0) best = INT_MAX, last_mass = -1;
  scan[tid] = local;
  __syncthreads();
  // exclusive prefix of the per-thread sums, in token order (serial per thread: 256 adds, fixed order)
  double run = before;
  for (int t = 0; t < tid; ++t) run += scan[t];
  int found = INT_MAX;
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    run += mass[e];
    if (found == INT_MAX && run > thr && mass[e] > 0.0) found = v0 + tid * kPer + e;
  }
  if (found != INT_MAX) atomicMin(&best, found);
  if (my_last >= 0) atomicMax(&last_mass, my_last);
  __syncthreads();
  if (tid == 0) p.next_token[nb] = best != INT_MAX ? best : last_mass;
}

template <bool BF16>
void launch_stats(const AcceptParams &p, bool vec, hipStream_t stream) {
  const dim3 grid(p.n_chunks, p.NB * (2 * p.K + 1));
  if (vec)
    hipLaunchKernelGGL((accept_stats_kernel<BF16, true>), grid, dim3(kThreads), 0, stream, p);
  else
    hipLaunchKernelGGL((accept_stats_kernel<BF16, false>), grid, dim3(kThreads), 0, stream, p);
}

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

size_t accept_workspace_bytes(int NB, int K, int V, int *chunk_out, int *n_chunks_out) {
  const int n_chunks = (V + kChunk - 1) / kChunk;
  if (chunk_out) *chunk_out = kChunk;
  if (n_chunks_out) *n_chunks_out = n_chunks;
  size_t b = 0;
  b += align_up((size_t)NB * (2 * K + 1) * n_chunks * 2 * sizeof(float));  // stats
  b += align_up((size_t)NB * sizeof(int32_t));                             // n_acc
  b += align_up((size_t)NB * 2 * n_chunks * sizeof(double));               // zsum
  b += align_up((size_t)NB * 2 * n_chunks * sizeof(double));               // rsum
  b += align_up((size_t)NB * 2 * sizeof(float));                           // rowmax
  return b;
}

void accept_carve_workspace(AcceptParams &p, void *ws) {
  uint8_t *at = (uint8_t *)ws;
  p.stats = (float *)at;
  at += align_up((size_t)p.NB * (2 * p.K + 1) * p.n_chunks * 2 * sizeof(float));
  p.n_acc = (int32_t *)at;
  at += align_up((size_t)p.NB * sizeof(int32_t));
  p.zsum = (double *)at;
  at += align_up((size_t)p.NB * 2 * p.n_chunks * sizeof(double));
  p.rsum = (double *)at;
  at += align_up((size_t)p.NB * 2 * p.n_chunks * sizeof(double));
  p.rowmax = (float *)at;
}

hipError_t launch_accept(const AcceptParams &p, hipStream_t stream) {
  const size_t esz = p.bf16 ? 2 : 4;
  const bool vec = ((size_t)p.V * esz) % 16 == 0;
  {
    ProfileScope scope(SLOT_ACCEPT_STATS, stream);
    if (p.bf16)
      launch_stats<true>(p, vec, stream);
    else
      launch_stats<false>(p, vec, stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  {
    ProfileScope scope(SLOT_ACCEPT_DECIDE, stream);
    hipLaunchKernelGGL(accept_decide_kernel, dim3(p.NB), dim3(64), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  {
    ProfileScope scope(SLOT_ACCEPT_RESID, stream);
    hipLaunchKernelGGL(accept_zsum_kernel, dim3(p.n_chunks, p.NB, 2), dim3(kThreads), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(accept_resid_kernel, dim3(p.n_chunks, p.NB), dim3(kThreads), 0, stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  {
    ProfileScope scope(SLOT_ACCEPT_PICK, stream);
    hipLaunchKernelGGL(accept_pick_kernel, dim3(p.NB), dim3(kThreads), 0, stream, p);
    return hipGetLastError();
  }
}

}  // namespace la
