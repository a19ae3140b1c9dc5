// Token-level speculative accept / resample over the vocabulary (gfx950).
//
// Section 2 ("Speculative Decoding"): the K drafted tokens of a branch are examined in
// order, x_i accepted with probability min(1, p_i(x_i)/q_i(x_i)); the first rejection n
// stops the walk and one token is drawn from norm(max(0, p_n - q_n)); with all K accepted
// a bonus token is drawn from p_K.
//
// Launches:
//   stats   one coalesced pass over every logit row (NB*(2K+1) rows x V): per (row, slice)
//           the exact maximum and sum 2^((x-max)*log2e/T), fp32.  This is the HBM-bound
//           part: each logit is read exactly once, 16-byte loads, eight in flight per lane.
//   decide  grid (fine slices, NB): every workgroup folds the slice statistics of its
//           branch, gathers p_i(x_i), q_i(x_i) and tests u*q < p in order (n); then the fp64
//           resampling path starts: its share of sum exp(z - max) of the two rows at
//           position n (target row n and draft row n, or target row K alone when n = K).
//   resid   grid (fine slices, NB): fp64 normalisers from the shares above, then per lane
//           the mass of its 8 consecutive tokens: max(0, p-q) (and p itself, which is the
//           distribution of the bonus token and the fallback when the residual has no
//           mass).  Per-lane and per-slice sums go to the workspace.
//   pick    grid NB: the slice in which the running sum first exceeds u_sample * total,
//           then the lane inside it (scan of the stored per-lane sums), then the token
//           among that lane's 8 (re-evaluated by one lane).
//   warp    (only with top-k / top-p) one workgroup per target row: the smallest logit the row keeps and the
//           mass of the kept tokens.  Both filters are predicates on a token's value (keep v iff fewer than k
//           tokens are larger; keep v iff the mass of the larger kept tokens is below top_p * Z_k), so equal
//           logits are never split.  With a small k, or with top-p alone, a bound taken from the lanes' largest
//           logits leaves a short list of candidate tokens, which is sorted and walked in descending order;
//           otherwise (and whenever such a list overflows or falls short) two radix selections over an
//           order-preserving key of the logit: the k-th largest by count, then among those the value at which
//           the descending cumulative mass reaches top_p of the kept mass.  decide / resid / pick then use
//           p(v) = [key(v) >= key_min] * exp((x_v - max)/T) / Z_kept for the target rows.
//   rowz    (only with top-p alone) grid (fine-slice groups, target rows): the fp64 mass of every target row in
//           fine slices, which warp folds: top-p's threshold is a share of the whole row's mass.
// The two resampling rows are re-read twice (2 of the 2K+1 rows of a branch; cache hits).
// fp64 there makes the blocked running sum agree with a sequential one to ~1e-16, so the
// drawn token does not depend on the summation order.
#include <limits.h>

#include "la_internal.hpp"

namespace la {
namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kThreads = 256;
constexpr int kFinePer = 8;                 // tokens per lane in the fp64 kernels (load_fine reads eight)
constexpr int kFine = kThreads * kFinePer;  // 2048 tokens per fine slice

// (bit-casting a vector element in place, __builtin_bit_cast(float, w[k]), reads element 0 with this compiler;
// pass the element by value instead)
__device__ __forceinline__ float as_f32(uint32_t w) { return __builtin_bit_cast(float, w); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xFFFF0000u); }

template <bool BF16>
__device__ __forceinline__ float load_logit(const void *base, size_t idx) {
  if constexpr (BF16) return __builtin_bit_cast(float, (uint32_t)((const uint16_t *)base)[idx] << 16);
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
template <bool BF16>
__device__ __forceinline__ const uint8_t *stacked_row(const AcceptParams &p, int rw) {
  constexpr size_t esz = BF16 ? 2 : 4;
  const int n_t = p.NB * (p.K + 1);
  if (rw < n_t) return (const uint8_t *)p.target + (size_t)rw * p.V * esz;
  return (const uint8_t *)p.draft + (size_t)(rw - n_t) * p.V * esz;
}

// ---------------------------------------------------------------------------------------------
// stats: grid (n_chunks, rows); a slice is 256 lanes x 8 16-byte loads (16384 bf16 / 8192 fp32 logits)
// ---------------------------------------------------------------------------------------------
template <bool BF16>
struct StatsShape {
  static constexpr int kLoads = 8;
  static constexpr int kPerVec = BF16 ? 8 : 4;
  static constexpr int kPer = kLoads * kPerVec;  // logits per lane
  static constexpr int kSlice = kThreads * kPer;
};

template <bool BF16, bool VEC>
__global__ __launch_bounds__(kThreads, 6) void accept_stats_kernel(const AcceptParams p) {
  using Sh = StatsShape<BF16>;
  __shared__ float red[2][kThreads / 64];
  const int c = blockIdx.x, rw = blockIdx.y;
  const int tid = threadIdx.x;
  const uint8_t *row = stacked_row<BF16>(p, rw);
  const int v0 = c * Sh::kSlice;
  const int v1 = min(p.V, v0 + Sh::kSlice);

  float x[Sh::kPer];
  if constexpr (VEC) {
    u32x4 w[Sh::kLoads];
#pragma unroll
    for (int e = 0; e < Sh::kLoads; ++e) {
      const int v = v0 + (e * kThreads + tid) * Sh::kPerVec;  // consecutive lanes read consecutive 16 B
      // V % kPerVec == 0 on this path, so a vector is all-in or all-out; out-of-range lanes re-read the row start
      w[e] = *(const u32x4 *)(row + (size_t)(v < v1 ? v : 0) * (BF16 ? 2 : 4));
    }
#pragma unroll
    for (int e = 0; e < Sh::kLoads; ++e) {
      const bool in = v0 + (e * kThreads + tid) * Sh::kPerVec < v1;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t word = w[e][k];
        if constexpr (BF16) {
          x[e * 8 + 2 * k] = in ? bf16_lo(word) : -INFINITY;
          x[e * 8 + 2 * k + 1] = in ? bf16_hi(word) : -INFINITY;
        } else {
          x[e * 4 + k] = in ? as_f32(word) : -INFINITY;
        }
      }
    }
  } else {
#pragma unroll
    for (int e = 0; e < Sh::kPer; ++e) {
      const int v = v0 + e * kThreads + tid;
      x[e] = v < v1 ? load_logit<BF16>(row, v) : -INFINITY;
    }
  }
  float m = x[0];
#pragma unroll
  for (int e = 1; e < Sh::kPer; ++e) m = fmaxf(m, x[e]);
  m = wave_max(m);
  if ((tid & 63) == 0) red[0][tid >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));  // slice maximum
  // a slice whose logits are all -inf (a masked part of the vocabulary) has mass 0: the exponent offset is taken
  // from 0 instead of from -inf, which would turn -inf - (-inf) into a NaN; the slice is recorded as (-inf, 0) and
  // drops out of every fold (weight 2^(-inf - row maximum) = 0)
  const float cm = -((m == -INFINITY) ? 0.f : m) * p.inv_temp_log2;
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < Sh::kPer; ++e) s += __builtin_amdgcn_exp2f(__builtin_fmaf(x[e], p.inv_temp_log2, cm));
  s = wave_sum(s);
  if ((tid & 63) == 0) red[1][tid >> 6] = s;
  __syncthreads();
  if (tid == 0) {
    f32x2 out = {m, (red[1][0] + red[1][1]) + (red[1][2] + red[1][3])};
    *(f32x2 *)(p.stats + ((size_t)rw * p.n_chunks + c) * 2) = out;
  }
}

// Fold the slice statistics of one row into its maximum and sum 2^((x-max)*c); called by a whole wavefront, lanes
// over slices, the same result in every lane.
__device__ __forceinline__ void wave_fold_row(const AcceptParams &p, int rw, int lane, float &m_out, float &z_out) {
  const float *st = p.stats + (size_t)rw * p.n_chunks * 2;
  float m = -INFINITY;
  for (int c = lane; c < p.n_chunks; c += 64) m = fmaxf(m, st[2 * c]);
  m = wave_max(m);
  float z = 0.f;
  for (int c = lane; c < p.n_chunks; c += 64)
    z += st[2 * c + 1] * __builtin_amdgcn_exp2f((st[2 * c] - m) * p.inv_temp_log2);
  m_out = m;
  z_out = wave_sum(z);
}

// Order-preserving key of an fp32 value: larger value <=> larger key (as unsigned).
__device__ __forceinline__ uint32_t order_key(float x) {
  const uint32_t b = __builtin_bit_cast(uint32_t, x + 0.0f);   // -0 and +0 are one value: (-0) + (+0) = +0
  return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

// exp(y) in fp64 for the arguments met here (y = (x - max)/T <= 0 up to rounding; the result only has to be the same
// function of y everywhere it is used, and within an ulp or two of the true value).  y = k ln2 + r with |r| <= ln2/2
// by a two-term reduction (k * ln2_hi is exact for |k| < 2^11), e^r by its Taylor polynomial of degree 13
// (remainder < 5e-18), then the scaling by 2^k, which also takes results below the normal range to denormals / zero.
// About 20 fp64 instructions, against several times that for the general library routine.
// a * b + c with the constant c read from scalar registers (left to itself the compiler copies every constant of the
// polynomial into a vector register pair first, two moves per step, to use the two-address form of the instruction)
__device__ __forceinline__ double fma_const(double a, double b, double c) {
  double d;
  asm("v_fma_f64 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "s"(c));
  return d;
}

__device__ __forceinline__ double exp64(double y) {
  y = fmax(y, -750.0);   // (y <= 0 up to rounding: x never exceeds the row maximum)
  // k = nearest integer to y * log2(e): adding 1.5 * 2^52 leaves it in the low bits of the sum (as a double by taking
  // the constant off again, as an integer in the low word of the bit pattern); the rounding and conversion
  // instructions this replaces run at a quarter of the rate of an addition
  const double shifted = __builtin_fma(y, 1.4426950408889634074, 6755399441055744.0);
  const double k = shifted - 6755399441055744.0;
  const int ki = (int)(uint32_t)__builtin_bit_cast(uint64_t, shifted);
  double r = __builtin_fma(-k, 6.93147180369123816490e-01, y);
  r = __builtin_fma(-k, 1.90821492927058770002e-10, r);
  double q = fma_const(r, 1.0 / 6227020800.0, 1.0 / 479001600.0);
  q = fma_const(q, r, 1.0 / 39916800.0);
  q = fma_const(q, r, 1.0 / 3628800.0);
  q = fma_const(q, r, 1.0 / 362880.0);
  q = fma_const(q, r, 1.0 / 40320.0);
  q = fma_const(q, r, 1.0 / 5040.0);
  q = fma_const(q, r, 1.0 / 720.0);
  q = fma_const(q, r, 1.0 / 120.0);
  q = fma_const(q, r, 1.0 / 24.0);
  q = fma_const(q, r, 1.0 / 6.0);
  q = __builtin_fma(q, r, 0.5);
  q = __builtin_fma(q, r, 1.0);
  q = __builtin_fma(q, r, 1.0);
  return __builtin_ldexp(q, ki);
}

// fp64 probability mass (unnormalised) of one logit: exp(x/T - max/T)
__device__ __forceinline__ double mass64(float x, double mx_over_t, double inv_temp) {
  return exp64((double)x * inv_temp - mx_over_t);
}

// The kFinePer consecutive logits of a row that a lane of the fp64 kernels owns, from token v (a multiple of
// kFinePer) on; tokens at or past V read as -inf.  vec: every row starts on a 16-byte boundary, so the eight values
// are one (bf16) or two (fp32) 16-byte loads.
template <bool BF16>
__device__ __forceinline__ void load_fine(const void *base, size_t row_off, int v, int V, bool vec, float (&x)[8]) {
  if (vec && v + 8 <= V) {
    if constexpr (BF16) {
      const u32x4 w = *(const u32x4 *)((const uint16_t *)base + row_off + v);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t word = w[k];
        x[2 * k] = bf16_lo(word);
        x[2 * k + 1] = bf16_hi(word);
      }
    } else {
      const u32x4 w0 = *(const u32x4 *)((const float *)base + row_off + v);
      const u32x4 w1 = *(const u32x4 *)((const float *)base + row_off + v + 4);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t a = w0[k], b = w1[k];
        x[k] = as_f32(a);
        x[4 + k] = as_f32(b);
      }
    }
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = v + e < V ? load_logit<BF16>(base, row_off + v + e) : -INFINITY;
  }
}

// ---------------------------------------------------------------------------------------------
// warp: grid NB*(K+1), one workgroup of 1024 lanes per target row (Section 4, Setup: temperature, top_k, top_p)
// ---------------------------------------------------------------------------------------------
constexpr int kWarpThreads = 1024;
constexpr int kRep = 16;   // histogram copies per workgroup
constexpr int kHist = 257; // elements between two copies: one more than the buckets, so that the same bucket of
                           // different copies lies in different LDS banks

// Calls f(x) for every logit of a row, the workgroup's lanes striding over it, with several loads in flight per
// lane (16-byte loads when the row allows: eight per lane and batch).
template <bool BF16, typename F>
__device__ __forceinline__ void row_foreach(const void *row, int V, F &&f) {
  constexpr int kPerVec = BF16 ? 8 : 4;
  constexpr int kInFlight = 8;   // 16-byte loads per lane and batch
  const int tid = threadIdx.x;
  if (V % kPerVec == 0) {   // then every row starts on a 16-byte boundary
    const int n_vec = V / kPerVec;
    for (int i0 = tid; i0 < n_vec; i0 += kInFlight * kWarpThreads) {
      u32x4 w[kInFlight];
#pragma unroll
      for (int j = 0; j < kInFlight; ++j) {
        const int i = i0 + j * kWarpThreads;
        w[j] = *(const u32x4 *)((const uint8_t *)row + (size_t)(i < n_vec ? i : i0) * 16);
      }
#pragma unroll
      for (int j = 0; j < kInFlight; ++j) {
        if (i0 + j * kWarpThreads >= n_vec) break;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const uint32_t word = w[j][k];
          if constexpr (BF16) {
            f(bf16_lo(word));
            f(bf16_hi(word));
          } else {
            f(as_f32(word));
          }
        }
      }
    }
  } else {
    for (int v0 = tid; v0 < V; v0 += 8 * kWarpThreads) {
      float x[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int v = v0 + j * kWarpThreads;
        x[j] = load_logit<BF16>(row, v < V ? v : v0);
      }
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (v0 + j * kWarpThreads < V) f(x[j]);
    }
  }
}

// Radix selection over the keys of a set of values, 8 bits per round from the top.  BY_MASS = false: the k-th
// largest key (count{key > result} < k <= count{key >= result}).  BY_MASS = true: the key at which the descending
// cumulative mass first reaches target (mass{key > result} < target <= mass{key >= result}); if the whole mass
// stays below target, floor_key.  BF16 values have 16 significant key bits: two rounds instead of four.
// `each(f)` calls f(x) for every value of the set, the workgroup's lanes sharing the work; values with a key below
// floor_key take no part (the caller guarantees that the answer lies at or above it).
// The mass histogram is accumulated in 64-bit fixed point (masses are at most 1, at most 2^21 of them; 40 fraction
// bits, each mass rounded to nearest): integer atomics add in any order to the same bits, so the selection is the
// same in every run, which floating-point atomics would not give.  The 2^-41 rounding per term moves a bucket's
// mass by a few 1e-10 of the row's mass at most, inside the margin within which a top-p decision counts as open.
template <bool BF16, bool BY_MASS, typename Each>
__device__ __forceinline__ uint32_t radix_select(Each &&each, double mx_over_t, double inv_temp, uint32_t floor_key,
                                                 int k, double target, uint32_t *cnt, double *mass,
                                                 uint32_t *s_pick, double *s_above) {
  constexpr int kRounds = BF16 ? 2 : 4;
  constexpr double kFix = 1099511627776.0;   // 2^40
  unsigned long long *imass = (unsigned long long *)mass;
  const int tid = threadIdx.x;
  uint32_t prefix = 0;          // the bits chosen so far (high bits of the key)
  double above = 0.0;           // BY_MASS: mass of the keys above the chosen prefix range
  int k_rem = k;
#pragma unroll 1
  for (int round = 0; round < kRounds; ++round) {
    const int shift = 24 - 8 * round;
    // kRep copies of the histogram, chosen by lane: the logits of a row crowd into a few of the 256 buckets of the
    // leading byte, and LDS serialises atomics of one instruction that hit the same address
    for (int i = tid; i < kHist * kRep; i += kWarpThreads) {
      if constexpr (BY_MASS)
        imass[i] = 0;
      else
        cnt[i] = 0;
    }
    __syncthreads();
    const int rep = (tid & (kRep - 1)) * kHist;
    each([&](float x) {
      const uint32_t key = order_key(x);
      const bool in_range = round == 0 || (key >> (shift + 8)) == (prefix >> (shift + 8));
      if (!in_range || key < floor_key) return;
      if constexpr (BY_MASS)
        atomicAdd(&imass[rep + ((key >> shift) & 255)],
                  (unsigned long long)__builtin_llrint(mass64(x, mx_over_t, inv_temp) * kFix));
      else
        atomicAdd(&cnt[rep + ((key >> shift) & 255)], 1u);
    });
    __syncthreads();
    if (tid < 256) {   // fold the copies, in order
      if constexpr (BY_MASS) {
        unsigned long long t = 0;
        for (int r = 0; r < kRep; ++r) t += imass[r * kHist + tid];
        imass[tid] = t;
      } else {
        uint32_t t = 0;
        for (int r = 0; r < kRep; ++r) t += cnt[r * kHist + tid];
        cnt[tid] = t;
      }
    }
    __syncthreads();
    if (tid == 0) {
      int pick = -1;
      if constexpr (BY_MASS) {
        double m = above;
        int lowest = -1;
        double low_mass = 0.0;
        for (int b = 255; b >= 0; --b) {
          if (imass[b] == 0) continue;
          const double mb = (double)imass[b] * (1.0 / kFix);
          if (m + mb >= target) {
            pick = b;
            break;
          }
          lowest = b, low_mass = mb;
          m += mb;
        }
        // below the first round the parent bucket did cross; if the running sum misses that by a rounding of its
        // additions, the crossing is in the lowest bucket with mass
        if (pick < 0 && round > 0) pick = lowest, m -= low_mass;
        *s_above = m;
      } else {
        int c = 0;
        for (int b = 255; b >= 0; --b) {
          if (c + (int)cnt[b] >= k_rem) {
            pick = b;
            k_rem -= c;
            break;
          }
          c += (int)cnt[b];
        }
        *s_above = (double)k_rem;
      }
      *s_pick = (uint32_t)pick;
    }
    __syncthreads();
    const uint32_t pick = *s_pick;
    if (pick == 0xFFFFFFFFu) return floor_key;   // BY_MASS only: the target lies beyond the whole mass
    prefix |= pick << shift;
    if constexpr (BY_MASS)
      above = *s_above;
    else
      k_rem = (int)*s_above;
    __syncthreads();
  }
  // a bf16 logit widened to fp32 has 16 zero low bits, which the key turns into 0xFFFF for negative values
  return BF16 ? (prefix | ((prefix >> 31) ? 0u : 0xFFFFu)) : prefix;
}

// Sum over the row of exp((x - max)/T) for keys >= floor_key, fp64, in a fixed order (per lane in token order, then
// a shuffle tree, then the wavefronts in order): the same value in every lane.
template <bool BF16>
__device__ __forceinline__ double kept_mass(const void *row, int V, double mx_over_t, double inv_temp,
                                            uint32_t floor_key, double *red, double *slot) {
  const int tid = threadIdx.x;
  double acc = 0.0;
  row_foreach<BF16>(row, V, [&](float x) {
    if (order_key(x) >= floor_key) acc += mass64(x, mx_over_t, inv_temp);
  });
  acc = wave_sum(acc);
  if ((tid & 63) == 0) red[tid >> 6] = acc;
  __syncthreads();
  if (tid == 0) {
    double t = 0.0;
    for (int w = 0; w < kWarpThreads / 64; ++w) t += red[w];
    *slot = t;
  }
  __syncthreads();
  const double out = *slot;
  __syncthreads();
  return out;
}

// The logit an order-preserving key came from.
__device__ __forceinline__ float key_value(uint32_t key) {
  return __builtin_bit_cast(float, (key >> 31) ? key ^ 0x80000000u : ~key);
}

constexpr int kSmallK = 128;   // largest top_k the candidate-list path takes
constexpr int kCand = 2048;    // its candidate list (LDS)

// The k-th largest of the workgroup's per-lane keys mk (k <= number of lanes), found bit by bit with ballot counts:
// the largest value lo such that at least k lanes have mk >= lo.  The same value in every lane.  One barrier per
// bit; s_cnt is scratch of 2 x (wavefronts) ints.
template <bool BF16>
__device__ __forceinline__ uint32_t kth_largest_lane_key(uint32_t mk, int k, int (*s_cnt)[kWarpThreads / 64]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t lo = 0;
  // (a bf16 logit's key has sixteen equal low bits, so its sixteen high bits decide)
  for (int bit = 31; bit >= (BF16 ? 16 : 0); --bit) {
    const uint32_t c = lo | (1u << bit);
    const int n_w = __popcll(__ballot(mk >= c));
    if (lane == 0) s_cnt[bit & 1][wave] = n_w;
    __syncthreads();
    int tot = 0;
#pragma unroll
    for (int w = 0; w < kWarpThreads / 64; ++w) tot += s_cnt[bit & 1][w];
    if (tot >= k) lo = c;
  }
  if (BF16 && !(lo >> 31)) lo |= 0xFFFFu;   // the low bits of a negative bf16 value's key: lo is that key itself
  return lo;
}

// Append `key` to list[] (capacity cap, length *n in LDS) for the lanes with take set: one LDS atomic per wavefront
// and call instead of one per lane.  *n counts every qualifying token, also past the capacity.
__device__ __forceinline__ void list_append(bool take, uint32_t key, uint32_t *list, int cap, int *n) {
  const uint64_t who = __ballot(take);
  if (!who) return;
  const int lane = threadIdx.x & 63, leader = __ffsll((unsigned long long)who) - 1;
  int base = 0;
  if (lane == leader) base = atomicAdd(n, __popcll(who));
  base = __shfl(base, leader);
  if (take) {
    const int i = base + __popcll(who & ((1ull << lane) - 1));
    if (i < cap) list[i] = key;
  }
}

// The tokens of a row with value >= lo_val appended to list[] as keys (see list_append), for bounds that about one
// token in a hundred reaches, so that nearly every wavefront-wide step of a plain scan would find one.  On 16-byte
// aligned rows a lane first marks the qualifying ones among the up to 64 tokens of its eight loads in a bit mask (one
// compare and one bit operation per token); then the marked tokens are appended in rounds, one per lane and round,
// their values read again (few, and just loaded).
template <bool BF16>
__device__ __forceinline__ void row_collect(const void *row, int V, float lo_val, uint32_t *list, int cap, int *n) {
  constexpr int kPerVec = BF16 ? 8 : 4;
  constexpr int kInFlight = 8;
  const int tid = threadIdx.x;
  if (V % kPerVec != 0) {
    row_foreach<BF16>(row, V, [&](float x) { list_append(x >= lo_val, order_key(x), list, cap, n); });
    return;
  }
  const int n_vec = V / kPerVec;
  for (int i0 = tid; i0 < n_vec; i0 += kInFlight * kWarpThreads) {
    u32x4 w[kInFlight];
#pragma unroll
    for (int j = 0; j < kInFlight; ++j) {
      const int i = i0 + j * kWarpThreads;
      w[j] = *(const u32x4 *)((const uint8_t *)row + (size_t)(i < n_vec ? i : i0) * 16);
    }
    uint64_t marks = 0;   // bit j*kPerVec + e: element e of load j qualifies
#pragma unroll
    for (int j = 0; j < kInFlight; ++j) {
      const bool in = i0 + j * kWarpThreads < n_vec;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t word = w[j][k];
        if constexpr (BF16) {
          if (in && bf16_lo(word) >= lo_val) marks |= 1ull << (j * 8 + 2 * k);
          if (in && bf16_hi(word) >= lo_val) marks |= 1ull << (j * 8 + 2 * k + 1);
        } else {
          if (in && as_f32(word) >= lo_val) marks |= 1ull << (j * 4 + k);
        }
      }
    }
    while (__ballot(marks != 0)) {
      const bool take = marks != 0;
      const int bit = take ? __ffsll((unsigned long long)marks) - 1 : 0;
      marks &= marks - 1;
      const int j = bit / kPerVec, e = bit - j * kPerVec;
      const size_t v = (size_t)(i0 + j * kWarpThreads) * kPerVec + e;
      const float x = take ? load_logit<BF16>(row, v) : 0.f;
      list_append(take, order_key(x), list, cap, n);
    }
  }
}

// The same for bounds that only a few dozen tokens of the row reach: a lane first takes the largest of the tokens of
// one 16-byte load; only when some lane of the wavefront has one at or above the bound are that load's tokens tested
// and appended one by one.
template <bool BF16>
__device__ __forceinline__ void row_collect_sparse(const void *row, int V, float lo_val, uint32_t *list, int cap,
                                                   int *n) {
  constexpr int kPerVec = BF16 ? 8 : 4;
  constexpr int kInFlight = 8;
  const int tid = threadIdx.x;
  if (V % kPerVec != 0) {
    row_foreach<BF16>(row, V, [&](float x) { list_append(x >= lo_val, order_key(x), list, cap, n); });
    return;
  }
  const int n_vec = V / kPerVec;
  for (int i0 = tid; i0 < n_vec; i0 += kInFlight * kWarpThreads) {
    u32x4 w[kInFlight];
#pragma unroll
    for (int j = 0; j < kInFlight; ++j) {
      const int i = i0 + j * kWarpThreads;
      w[j] = *(const u32x4 *)((const uint8_t *)row + (size_t)(i < n_vec ? i : i0) * 16);
    }
#pragma unroll
    for (int j = 0; j < kInFlight; ++j) {
      const bool in = i0 + j * kWarpThreads < n_vec;
      float x[kPerVec];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t word = w[j][k];
        if constexpr (BF16) {
          x[2 * k] = bf16_lo(word);
          x[2 * k + 1] = bf16_hi(word);
        } else {
          x[k] = as_f32(word);
        }
      }
      float top = x[0];
#pragma unroll
      for (int e = 1; e < kPerVec; ++e) top = fmaxf(top, x[e]);
      if (__ballot(in && top >= lo_val)) {
#pragma unroll
        for (int e = 0; e < kPerVec; ++e) list_append(in && x[e] >= lo_val, order_key(x[e]), list, cap, n);
      }
    }
  }
}

// Bitonic sort of list[0..n) in descending order, in place, by the whole workgroup; n <= kCand.  Entries n..N-1 (N
// the next power of two, at least 128) are filled with 0, which is below every key.  Compare-exchange steps whose
// partners are at least 128 apart involve the whole workgroup and end in a barrier; the steps below that stay inside
// 128-entry blocks, one block per wavefront and one comparator per lane, and need no barrier between them (a
// wavefront's LDS accesses are carried out in order).
__device__ __forceinline__ void sort_desc(uint32_t *list, int n) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int N = 128;
  while (N < n) N <<= 1;
  for (int i = n + threadIdx.x; i < N; i += kWarpThreads) list[i] = 0u;
  __syncthreads();
  auto exchange = [&](int i, int o, int k) {
    const uint32_t a = list[i], b = list[o];
    const bool desc = (i & k) == 0;
    if (desc ? a < b : a > b) list[i] = b, list[o] = a;
  };
  for (int k = 2; k <= N; k <<= 1) {
    int j = k >> 1;
    for (; j >= 128; j >>= 1) {
      for (int c = threadIdx.x; c < N / 2; c += kWarpThreads) {   // comparator c: a zero bit inserted at j
        const int i = ((c & ~(j - 1)) << 1) | (c & (j - 1));
        exchange(i, i | j, k);
      }
      __syncthreads();
    }
    if (wave * 128 < N) {
      for (; j > 0; j >>= 1) {
        const int i = wave * 128 + (((lane & ~(j - 1)) << 1) | (lane & (j - 1)));
        exchange(i, i | j, k);
        __builtin_amdgcn_wave_barrier();
      }
    }
    __syncthreads();
  }
}

// Sort the n <= kCand keys of cand[] into sorted[] in descending order by rank counting (equal keys are the same
// value, so their mutual order does not matter) and put the exact fp64 mass of sorted[i] into cmass[i].
__device__ __forceinline__ void sort_list_with_masses(const uint32_t *cand, int n, uint32_t *sorted, double *cmass,
                                                      double mx_over_t, double inv_temp) {
  for (int i = threadIdx.x; i < n; i += kWarpThreads) {
    const uint32_t ki = cand[i];
    int rank = 0;
    for (int j = 0; j < n; ++j) {
      const uint32_t kj = cand[j];
      rank += (kj > ki || (kj == ki && j < i)) ? 1 : 0;
    }
    sorted[rank] = ki;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < n; i += kWarpThreads) cmass[i] = mass64(key_value(sorted[i]), mx_over_t, inv_temp);
  __syncthreads();
}

// top-k with a small k, then top-p, in two passes over the row and without a histogram.  Pass 1: every lane keeps
// the largest key among its tokens; the k-th largest of these lane maxima (found bit by bit with ballot counts) is a
// lower bound of the row's k-th largest key, because at least k tokens reach it.  Pass 2: the keys at or above that
// bound go to a list in LDS (a few dozen for random logits; when more than kCand qualify, e.g. a row of equal
// logits, the caller takes the histogram path instead: returns false, the same decision in every lane).  The list is
// sorted by rank counting (the order of equal keys does not matter: they are the same value), and one lane walks it
// in descending order exactly as the definition reads: the tokens down to the k-th largest value stay, Z_k is their
// mass, then value groups are taken while the mass above them is below top_p * Z_k.
template <bool BF16>
__device__ __forceinline__ bool warp_small_k(const AcceptParams &p, const void *row, uint32_t *cand, uint32_t *sorted,
                                             double *cmass, float *row_max_out, uint32_t *key_min_out,
                                             double *z_out) {
  __shared__ int s_cnt[2][kWarpThreads / 64];
  __shared__ float s_wmax[kWarpThreads / 64];
  __shared__ int s_n;
  __shared__ uint32_t s_key;
  __shared__ double s_z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int k = p.top_k;
  float mx = -INFINITY;   // a lane without tokens counts as holding -inf
  row_foreach<BF16>(row, p.V, [&](float x) { mx = fmaxf(mx, x); });
  const uint32_t mk = order_key(mx);
  {   // the row maximum falls out of the same pass (made visible by the first barrier of the search below)
    const float wm = wave_max(mx);
    if (lane == 0) s_wmax[wave] = wm;
  }
  const uint32_t lo = kth_largest_lane_key<BF16>(mk, k, s_cnt);   // k <= kSmallK < the number of lanes
  float row_max = s_wmax[0];
#pragma unroll
  for (int w = 1; w < kWarpThreads / 64; ++w) row_max = fmaxf(row_max, s_wmax[w]);
  *row_max_out = row_max;
  const double mx_over_t = (double)row_max * p.inv_temp;
  const float lo_val = key_value(lo);        // the k-th largest lane maximum (-inf when fewer than k lanes own a token)
  if (tid == 0) s_n = 0;
  __syncthreads();
  // comparing the values is comparing the keys (no NaNs; -0 == +0 on both sides)
  row_collect_sparse<BF16>(row, p.V, lo_val, cand, kCand, &s_n);
  __syncthreads();
  const int n_c = s_n;   // >= k
  if (n_c > kCand) return false;
  sort_list_with_masses(cand, n_c, sorted, cmass, mx_over_t, p.inv_temp);
  const uint32_t kth = sorted[k - 1];
  if (n_c <= 64) {
    // the usual case: the whole list fits one wavefront, lane j holding the j-th largest key and its mass
    if (wave == 0) {
      const bool in = lane < n_c;
      const uint32_t key = in ? sorted[lane] : 0u;
      const bool by_k = in && key >= kth;                 // kept by top-k: a leading part of the lanes
      const double mj = by_k ? cmass[lane] : 0.0;
      const uint64_t kmask = __ballot(by_k);
      int kept = __popcll(kmask);
      if (p.top_p < 1.0f) {
        const double zk = wave_sum(mj);
        const double target = (double)p.top_p * zk;
        double incl = mj;                                   // inclusive running mass in descending order
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
          const double up = __shfl_up(incl, off);
          if (lane >= off) incl += up;
        }
        const double before = __shfl_up(incl, 1);
        const double excl = lane ? before : 0.0;
        // mass above a token = running mass before the first lane of its value group
        const uint32_t prev_key = __shfl_up(key, 1);
        const uint64_t starts = __ballot(lane == 0 || key != prev_key);
        const uint64_t upto = starts & (lane == 63 ? ~0ull : ((2ull << lane) - 1));
        const int g = 63 - __clzll((long long)upto);
        const double above = __shfl(excl, g);
        kept = __popcll(__ballot(by_k && above < target));   // a leading part as well: `above` never falls
      }
      const double z = wave_sum(lane < kept ? mj : 0.0);
      const uint32_t key_last = __shfl(key, kept - 1);
      if (lane == 0) s_key = key_last, s_z = z;
    }
  } else if (tid == 0) {
    int n_k = k;
    while (n_k < n_c && sorted[n_k] == kth) ++n_k;   // ties with the k-th largest stay
    int kept = n_k;
    if (p.top_p < 1.0f) {
      double zk = 0.0;
      for (int j = 0; j < n_k; ++j) zk += cmass[j];
      const double target = (double)p.top_p * zk;
      double above = 0.0;
      int j = 0;
      while (j < n_k && above < target) {   // the tokens of one value stay or go together
        int e = j;
        double group = 0.0;
        while (e < n_k && sorted[e] == sorted[j]) group += cmass[e++];
        above += group;
        j = e;
      }
      kept = j;
    }
    double z = 0.0;
    for (int j = 0; j < kept; ++j) z += cmass[j];
    s_key = sorted[kept - 1];
    s_z = z;
  }
  __syncthreads();
  *key_min_out = s_key;
  *z_out = s_z;
  return true;
}

// top-p without top-k through a candidate list.  zk, the exact fp64 mass of the whole row, is the fold of the row's
// fine-slice sums (accept_rowz_kernel).  One pass gives every lane's largest logit.  The kListRank-th largest of the
// lane maxima is a value that a bounded number of tokens reach (a rank statistic: about 1400 of a long row whatever
// the logits' law, when tokens of all sizes are spread evenly over the lanes); the tokens at or above it are listed
// in a second pass, sorted, given their exact masses, and the kept set is read off the list as the definition says:
// value groups in descending order while the mass above them is below top_p * zk.  The list is checked exactly: it
// must hold at least top_p * zk (then every token outside it has at least that much mass above it and is dropped).
// When it does not, or when more than kCand tokens qualify, the caller takes the histogram path (returns false, the
// same in every lane); zk is returned in either case.
constexpr int kListRank = 768;

template <bool BF16>
__device__ __forceinline__ bool warp_top_p_list(const AcceptParams &p, const void *row, const double *zs,
                                                double mx_over_t, double *red, uint32_t *list, double *cmass,
                                                double *zk_out, uint32_t *key_min_out, double *z_out) {
  __shared__ int s_cnt[2][kWarpThreads / 64];
  __shared__ int s_n, s_ok;
  __shared__ uint32_t s_key;
  __shared__ double s_z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float mx = -INFINITY;
  row_foreach<BF16>(row, p.V, [&](float x) { mx = fmaxf(mx, x); });
  // zk from the row's fine-slice sums (accept_rowz_kernel), in a fixed order: slice t in lane t, a butterfly per
  // wavefront, the wavefronts in order
  double acc = 0.0;
  for (int t = tid; t < p.n_fine; t += kWarpThreads) acc += zs[t];
  acc = wave_sum(acc);
  if (lane == 0) red[wave] = acc;
  const uint32_t lo = kth_largest_lane_key<BF16>(order_key(mx), kListRank, s_cnt);   // (its barriers publish red[])
  double zk = 0.0;
#pragma unroll
  for (int w = 0; w < kWarpThreads / 64; ++w) zk += red[w];
  *zk_out = zk;
  const float lo_val = key_value(lo);   // -inf when fewer than kListRank lanes own a token: the whole row is listed
  if (tid == 0) s_n = 0;
  __syncthreads();
  row_collect<BF16>(row, p.V, lo_val, list, kCand, &s_n);
  __syncthreads();
  const int n_c = s_n;
  if (n_c > kCand || n_c < 1) return false;
  sort_desc(list, n_c);
  for (int i = tid; i < n_c; i += kWarpThreads) cmass[i] = mass64(key_value(list[i]), mx_over_t, p.inv_temp);
  __syncthreads();
  if (wave == 0) {
    // lane l owns the list entries [l*per, (l+1)*per); running masses in descending order of the keys
    const double target = (double)p.top_p * zk;
    const int per = (n_c + 63) / 64;
    const int i0 = min(n_c, lane * per), i1 = min(n_c, i0 + per);
    double own = 0.0;
    for (int i = i0; i < i1; ++i) own += cmass[i];
    double incl = own;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const double up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    const double total = __shfl(incl, 63);
    const double before = __shfl_up(incl, 1);
    // first entry with at least `target` of mass before it (n_c if none): the entries before it stay whatever
    // their value groups; if it lies inside a value group, that group stays as a whole
    double run = lane ? before : 0.0;
    int cross = INT_MAX;
    for (int i = i0; i < i1; ++i) {
      if (cross == INT_MAX && !(run < target)) cross = i;
      run += cmass[i];
    }
    const uint64_t hits = __ballot(cross != INT_MAX);
    int first = n_c;
    if (hits) first = __shfl(cross, __ffsll((unsigned long long)hits) - 1);
    const uint32_t kref = list[first - 1];   // first >= 1: nothing lies before entry 0
    int end = INT_MAX;
    for (int i = max(i0, first); i < i1; ++i)
      if (end == INT_MAX && list[i] != kref) end = i;
    const uint64_t ends = __ballot(end != INT_MAX);
    int kept = n_c;
    if (ends) kept = __shfl(end, __ffsll((unsigned long long)ends) - 1);
    double zl = 0.0;
    for (int i = i0; i < min(i1, kept); ++i) zl += cmass[i];
    const double z = wave_sum(zl);
    if (lane == 0) {
      s_ok = total >= target ? 1 : 0;   // otherwise the kept set continues below the listed tokens
      s_key = list[kept - 1];
      s_z = z;
    }
  }
  __syncthreads();
  if (!s_ok) return false;
  *key_min_out = s_key;
  *z_out = s_z;
  return true;
}

// rowz: grid (groups of kRowzGroup fine slices, NB*(K+1)).  fp64 sum of exp((x - max)/T) over each 2048-token fine
// slice of one target row, for top-p without top-k, whose threshold is a share of the row's whole mass: the row's
// exponentials are spread over the chip here instead of being one workgroup's pass in the warp kernel.  A workgroup
// takes several slices so that its start-up (the row maximum from the slice statistics) is shared and all its loads
// are in flight together.
constexpr int kRowzGroup = 4;

template <bool BF16>
__global__ __launch_bounds__(kThreads) void accept_rowz_kernel(const AcceptParams p) {
  __shared__ float s_wm[kThreads / 64];
  __shared__ double red[kRowzGroup][kThreads / 64];
  const int c0 = blockIdx.x * kRowzGroup, rw = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  // the row maximum from the slice statistics (exact, so the same value in every workgroup and in the warp kernel)
  const float *st = p.stats + (size_t)rw * p.n_chunks * 2;
  float m = -INFINITY;
  for (int ch = tid; ch < p.n_chunks; ch += kThreads) m = fmaxf(m, st[2 * ch]);
  m = wave_max(m);
  if (lane == 0) s_wm[wave] = m;
  const bool vec = ((size_t)p.V * (BF16 ? 2 : 4)) % 16 == 0;
  float x[kRowzGroup][kFinePer];
#pragma unroll
  for (int g = 0; g < kRowzGroup; ++g)   // (slices past the row read as -inf)
    load_fine<BF16>(p.target, (size_t)rw * p.V, (c0 + g) * kFine + tid * kFinePer, p.V, vec, x[g]);
  __syncthreads();
  m = fmaxf(fmaxf(s_wm[0], s_wm[1]), fmaxf(s_wm[2], s_wm[3]));
  const double mx_over_t = (double)m * p.inv_temp;
#pragma unroll
  for (int g = 0; g < kRowzGroup; ++g) {
    double acc = 0.0;
#pragma unroll
    for (int e = 0; e < kFinePer; ++e) acc += mass64(x[g][e], mx_over_t, p.inv_temp);   // (past V: -inf, mass 0)
    acc = wave_sum(acc);
    if (lane == 0) red[g][wave] = acc;
  }
  __syncthreads();
  if (tid < kRowzGroup && c0 + tid < p.n_fine)
    p.warp_zs[(size_t)rw * p.n_fine + c0 + tid] = (red[tid][0] + red[tid][1]) + (red[tid][2] + red[tid][3]);
}

template <bool BF16>
__global__ __launch_bounds__(kWarpThreads) void accept_warp_kernel(const AcceptParams p) {
  __shared__ double mass[kHist * kRep];               // the count histogram shares this storage
  uint32_t *cnt = (uint32_t *)mass;
  __shared__ uint32_t s_pick;
  __shared__ double s_above, s_slot;
  __shared__ double red[kWarpThreads / 64];
  __shared__ float s_m;
  const int rw = blockIdx.x;   // target row nb*(K+1) + i
  const int tid = threadIdx.x;
  const uint8_t *row = (const uint8_t *)p.target + (size_t)rw * p.V * (BF16 ? 2 : 4);
  auto each_of_row = [&](auto &&f) { row_foreach<BF16>(row, p.V, f); };
  uint32_t key_min = 0;
  double zw = 0.0;
  float m = 0.f;
  bool done = false;
  if (p.top_k > 0 && p.top_k < p.V && p.top_k <= kSmallK)   // the candidate list lives in the histogram's storage
    done = warp_small_k<BF16>(p, row, cnt, cnt + kCand, mass + kCand, &m, &key_min, &zw);
  if (!done) {
    if (tid < 64) {
      float z;
      wave_fold_row(p, rw, tid, m, z);
      if (tid == 0) s_m = m;
    }
    __syncthreads();
    m = s_m;
    const double mx_over_t = (double)m * p.inv_temp;
    key_min = 0;
    const bool use_k = p.top_k > 0 && p.top_k < p.V;
    if (use_k)
      key_min = radix_select<BF16, false>(each_of_row, 0.0, 0.0, 0u, p.top_k, 0.0, cnt, mass, &s_pick, &s_above);
    bool listed = false;
    if (p.top_p < 1.0f) {
      double zk = 0.0;
      if (!use_k)   // (the candidate list lives in the histogram's storage)
        listed = warp_top_p_list<BF16>(p, row, p.warp_zs + (size_t)rw * p.n_fine, mx_over_t, red, cnt, mass + kCand,
                                       &zk, &key_min, &zw);
      else
        zk = kept_mass<BF16>(row, p.V, mx_over_t, p.inv_temp, key_min, red, &s_slot);
      if (!listed)
        key_min = radix_select<BF16, true>(each_of_row, mx_over_t, p.inv_temp, key_min, 0, (double)p.top_p * zk, cnt,
                                           mass, &s_pick, &s_above);
    }
    if (!listed) zw = kept_mass<BF16>(row, p.V, mx_over_t, p.inv_temp, key_min, red, &s_slot);
  }
  if (tid == 0) {
    p.warp_key[rw] = key_min;
    p.warp_z[rw] = zw;
    p.warp_max[rw] = m;
  }
}

// ---------------------------------------------------------------------------------------------
// decide: grid (n_fine, NB).  Accepted length of the branch (every workgroup derives it; slice 0 publishes it),
// then this slice's share of the fp64 normalisers of the resampling rows.
// ---------------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(kThreads) void accept_decide_kernel(const AcceptParams p) {
  constexpr int kPass = 64;                       // drafted positions examined per pass
  constexpr int kStage = 2048;                    // slice statistics (max, sum) staged in LDS per pass
  __shared__ float sm[2][kPass], sz[2][kPass];    // [target|draft][position in pass]: folded row statistics
  __shared__ f32x2 s_stat[kStage];
  __shared__ float s_top[2];                      // maxima of the resampling rows
  __shared__ float s_bonus;                       // maximum of target row K
  __shared__ int s_first, s_have_bonus;
  __shared__ double red[2][kThreads / 64];
  const int c = blockIdx.x, nb = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n_t = p.NB * (p.K + 1);
  const int n_which = p.draft ? 2 : 1;   // point-mass draft: there are no draft rows
  if (tid == 0) s_first = p.K, s_have_bonus = 0;
  __syncthreads();
  int i0 = 0;
  bool have_top = false;
  for (; i0 < p.K; i0 += kPass) {   // a later pass cannot lower the first rejection found in an earlier one
    const int cnt = min(kPass, p.K - i0);
    // what a position's test needs from global memory besides the row statistics; issued first so that the two
    // dependent round trips (token, then its two logits) overlap the fold below
    int x = 0;
    float tx = 0.f, dx = 0.f, u = 0.f;
    if (tid < cnt) {
      const int i = i0 + tid;
      x = p.tokens[(size_t)nb * p.K + i];
      u = p.u_accept[(size_t)nb * p.K + i];
      tx = load_logit<BF16>(p.target, ((size_t)nb * (p.K + 1) + i) * p.V + x);
      if (p.draft) dx = load_logit<BF16>(p.draft, ((size_t)nb * p.K + i) * p.V + x);
    }
    // rows folded in this pass: cnt target rows, cnt draft rows and, in the last pass, target row K (the bonus row)
    const int bonus = i0 + cnt == p.K ? 1 : 0;
    const int n_rows = n_which * cnt + bonus;
    auto row_of = [&](int slot) {
      if (slot == n_which * cnt) return nb * (p.K + 1) + p.K;
      const int which = slot >= cnt, j = slot - which * cnt;
      return which ? n_t + nb * p.K + i0 + j : nb * (p.K + 1) + i0 + j;
    };
    if (n_rows * p.n_chunks <= kStage) {
      // all slice statistics in one round of loads, then one lane per row folds its slices from LDS
      for (int idx = tid; idx < n_rows * p.n_chunks; idx += kThreads) {
        const int slot = idx / p.n_chunks, ch = idx - slot * p.n_chunks;
        s_stat[idx] = *(const f32x2 *)(p.stats + ((size_t)row_of(slot) * p.n_chunks + ch) * 2);
      }
      __syncthreads();
      if (tid < n_rows) {
        const f32x2 *st = s_stat + tid * p.n_chunks;
        float m = -INFINITY;
        for (int ch = 0; ch < p.n_chunks; ++ch) m = fmaxf(m, st[ch][0]);
        float z = 0.f;
        for (int ch = 0; ch < p.n_chunks; ++ch)
          z += st[ch][1] * __builtin_amdgcn_exp2f((st[ch][0] - m) * p.inv_temp_log2);
        if (tid == n_which * cnt) {
          s_bonus = m;
          s_have_bonus = 1;
        } else {
          const int which = tid >= cnt, j = tid - which * cnt;
          sm[which][j] = m, sz[which][j] = z;
        }
      }
    } else {
      for (int slot = wave; slot < n_which * cnt; slot += kThreads / 64) {   // wavefront per row
        const int which = slot >= cnt, j = slot - which * cnt;
        float m, z;
        wave_fold_row(p, row_of(slot), lane, m, z);
        if (lane == 0) sm[which][j] = m, sz[which][j] = z;
      }
    }
    __syncthreads();
    if (tid < cnt) {
      const int i = i0 + tid;
      float px = __builtin_amdgcn_exp2f((tx - sm[0][tid]) * p.inv_temp_log2) / sz[0][tid];
      if (p.warp_key) {  // warped target: x has mass only if its row keeps it, normalised by the kept mass
        const int wr = nb * (p.K + 1) + i;
        px = order_key(tx) >= p.warp_key[wr]
                 ? __builtin_amdgcn_exp2f((tx - sm[0][tid]) * p.inv_temp_log2) / (float)p.warp_z[wr]
                 : 0.f;
      }
      float qx = 1.0f;   // point-mass draft at x
      if (p.draft) qx = __builtin_amdgcn_exp2f((dx - sm[1][tid]) * p.inv_temp_log2) / sz[1][tid];
      if (!(u * qx < px)) atomicMin(&s_first, i);
      if (c == 0 && p.ratio) p.ratio[(size_t)nb * p.K + i] = px / qx;
    }
    __syncthreads();
    if (s_first < p.K) {  // uniform: the first rejection lies in this pass
      // exact maxima of the resampling rows: target row n and draft row n, both folded in this pass
      if (!have_top && tid == 0) s_top[0] = sm[0][s_first - i0], s_top[1] = p.draft ? sm[1][s_first - i0] : 0.f;
      have_top = true;
      // the workgroup that reports the ratios goes on through the remaining passes (every position gets its ratio,
      // also those behind the rejection); s_first cannot change any more, atomicMin only lowers it to values < i
      if (!(c == 0 && p.ratio)) break;
    }
    __syncthreads();  // sm / sz free for the next pass
  }
  const int n = s_first;
  // everything accepted: the maximum of target row K alone
  if (n < p.K) {
    // s_top was set in the pass that found n
  } else if (s_have_bonus) {
    if (tid == 0) s_top[0] = s_bonus, s_top[1] = 0.f;
  } else if (wave == 0) {
    float m, z;
    wave_fold_row(p, nb * (p.K + 1) + p.K, lane, m, z);
    if (lane == 0) s_top[0] = m, s_top[1] = 0.f;
  }
  __syncthreads();
  const float mt = s_top[0], mq = s_top[1];
  if (c == 0 && tid == 0) {
    p.accepted_len[nb] = n;
    p.n_acc[nb] = n;
    p.rowmax[2 * nb] = mt;
    p.rowmax[2 * nb + 1] = mq;
  }
  const int v0 = c * kFine;
  const size_t trow = ((size_t)nb * (p.K + 1) + n) * p.V;
  const size_t drow = ((size_t)nb * p.K + (n < p.K ? n : 0)) * p.V;
  const double mt_t = (double)mt * p.inv_temp, mq_t = (double)mq * p.inv_temp;
  double st = 0.0, sq = 0.0;
  const bool vec = ((size_t)p.V * (BF16 ? 2 : 4)) % 16 == 0;
  const bool with_draft = n < p.K && p.draft;
  const int vb = v0 + tid * kFinePer;
  float tx[kFinePer], dx[kFinePer];
  load_fine<BF16>(p.target, trow, vb, p.V, vec, tx);
  if (with_draft) load_fine<BF16>(p.draft, drow, vb, p.V, vec, dx);
#pragma unroll
  // no bounds test per token: load_fine gives -inf past V, whose mass is exactly 0, and the eight exponentials of a
  // lane can then be evaluated side by side instead of one dependent chain after the other
  for (int e = 0; e < kFinePer; ++e) {
    st += mass64(tx[e], mt_t, p.inv_temp);
    if (with_draft) sq += mass64(dx[e], mq_t, p.inv_temp);
  }
  st = wave_sum(st);
  sq = wave_sum(sq);
  if ((tid & 63) == 0) red[0][tid >> 6] = st, red[1][tid >> 6] = sq;
  __syncthreads();
  if (tid == 0) {
    p.zsum[((size_t)nb * 2 + 0) * p.n_fine + c] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
    p.zsum[((size_t)nb * 2 + 1) * p.n_fine + c] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
  }
}

constexpr int kMaxFine = 1024;   // fine slices per row the fp64 kernels can stage in LDS (vocab <= 2M)

// Two rows of n <= kMaxFine doubles each, folded together so that their loads are one round trip.  load: a lane's
// terms (index tid + kThreads*j) into registers.  sum: the two sums, the same values in every lane of the workgroup
// and in every workgroup that folds the same terms (fixed association: per lane its terms in index order, a
// butterfly inside each wavefront, the wavefronts in order); with buf0 / buf1 given the terms are also left there.
struct FoldPair {
  double a[kMaxFine / kThreads], b[kMaxFine / kThreads];
  __device__ __forceinline__ void load(const double *v0, const double *v1, int n) {
#pragma unroll
    for (int j = 0; j < kMaxFine / kThreads; ++j) {
      const int c = threadIdx.x + kThreads * j;
      a[j] = c < n ? v0[c] : 0.0;
      b[j] = c < n ? v1[c] : 0.0;
    }
  }
  __device__ __forceinline__ void sum(int n, double *buf0, double *buf1, double *s0, double *s1) const {
    __shared__ double fold_red[2][kThreads / 64];
    double x = 0.0, y = 0.0;
#pragma unroll
    for (int j = 0; j < kMaxFine / kThreads; ++j) {
      const int c = threadIdx.x + kThreads * j;
      if (c < n) {
        if (buf0) buf0[c] = a[j];
        if (buf1) buf1[c] = b[j];
        x += a[j];
        y += b[j];
      }
    }
    x = wave_sum(x);
    y = wave_sum(y);
    __syncthreads();   // fold_red free again (a previous call's readers are past their reads)
    if ((threadIdx.x & 63) == 0) fold_red[0][threadIdx.x >> 6] = x, fold_red[1][threadIdx.x >> 6] = y;
    __syncthreads();
    *s0 = (fold_red[0][0] + fold_red[0][1]) + (fold_red[0][2] + fold_red[0][3]);
    *s1 = (fold_red[1][0] + fold_red[1][1]) + (fold_red[1][2] + fold_red[1][3]);
  }
};

// residual mass and target mass of the tokens of branch nb at position n, fp64
template <bool BF16>
struct ResidCtx {
  const void *target, *draft;
  size_t trow, drow;
  double mt, mq, inv_zt, inv_zq, inv_temp;   // maxima over T, reciprocals of the normalisers, 1/T
  bool has_draft;
  int removed;   // point-mass draft after a rejection: the drafted token, which has no residual mass; else -1
  uint32_t key_min;   // warped target: smallest key the row keeps (0: everything)
  // tx, dx: the target and draft logit of token v (dx is read only with a draft row)
  __device__ __forceinline__ void eval(int v, float tx, float dx, double &r, double &pm) const {
    pm = order_key(tx) >= key_min ? mass64(tx, mt, inv_temp) * inv_zt : 0.0;
    r = v == removed ? 0.0 : pm;
    if (has_draft) {
      const double qm = mass64(dx, mq, inv_temp) * inv_zq;
      r = pm - qm;
      if (r < 0.0) r = 0.0;
    }
  }
};

template <bool BF16>
__device__ __forceinline__ ResidCtx<BF16> make_ctx(const AcceptParams &p, int nb) {
  ResidCtx<BF16> x;
  FoldPair zs;   // the slice shares of the two normalisers: requested together with everything else below
  zs.load(p.zsum + ((size_t)nb * 2 + 0) * p.n_fine, p.zsum + ((size_t)nb * 2 + 1) * p.n_fine, p.n_fine);
  const int n = p.n_acc[nb];
  x.target = p.target;
  x.draft = p.draft;
  x.trow = ((size_t)nb * (p.K + 1) + n) * p.V;
  x.has_draft = n < p.K && p.draft;
  x.removed = (n < p.K && !p.draft) ? p.tokens[(size_t)nb * p.K + n] : -1;
  x.drow = x.has_draft ? ((size_t)nb * p.K + n) * p.V : 0;
  x.inv_temp = p.inv_temp;
  x.mt = (double)p.rowmax[2 * nb] * p.inv_temp;
  x.mq = (double)p.rowmax[2 * nb + 1] * p.inv_temp;
  double zt, zq;
  zs.sum(p.n_fine, nullptr, nullptr, &zt, &zq);
  if (!x.has_draft) zq = 1.0;
  x.key_min = 0;
  if (p.warp_key) {   // the kept mass replaces the row's full normaliser
    x.key_min = p.warp_key[nb * (p.K + 1) + n];
    zt = p.warp_z[nb * (p.K + 1) + n];
  }
  x.inv_zt = 1.0 / zt;
  x.inv_zq = 1.0 / zq;
  return x;
}

// ---------------------------------------------------------------------------------------------
// resid: grid (n_fine, NB): per-lane and per-slice fp64 sums of the residual and of p
// ---------------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(kThreads) void accept_resid_kernel(const AcceptParams p) {
  __shared__ double red[2][kThreads / 64];
  const int c = blockIdx.x, nb = blockIdx.y, tid = threadIdx.x;
  const ResidCtx<BF16> ctx = make_ctx<BF16>(p, nb);
  const int v0 = c * kFine;
  double sr = 0.0, sp = 0.0;
  const bool vec = ((size_t)p.V * (BF16 ? 2 : 4)) % 16 == 0;
  const int vb = v0 + tid * kFinePer;
  float tx[kFinePer], dx[kFinePer];
  load_fine<BF16>(ctx.target, ctx.trow, vb, p.V, vec, tx);
  if (ctx.has_draft) load_fine<BF16>(ctx.draft, ctx.drow, vb, p.V, vec, dx);
#pragma unroll
  for (int e = 0; e < kFinePer; ++e) {   // (past V: -inf, no mass of either kind)
    double r, pm;
    ctx.eval(vb + e, tx[e], ctx.has_draft ? dx[e] : 0.f, r, pm);
    sr += r;
    sp += pm;
  }
  double *ls = p.lane_sums + (((size_t)nb * p.n_fine + c) * kThreads + tid) * 2;
  ls[0] = sr;
  ls[1] = sp;
  sr = wave_sum(sr);
  sp = wave_sum(sp);
  if ((tid & 63) == 0) red[0][tid >> 6] = sr, red[1][tid >> 6] = sp;
  __syncthreads();
  if (tid == 0) {
    p.rsum[((size_t)nb * 2 + 0) * p.n_fine + c] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
    p.rsum[((size_t)nb * 2 + 1) * p.n_fine + c] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
  }
}

// ---------------------------------------------------------------------------------------------
// pick: grid NB
// ---------------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(kThreads) void accept_pick_kernel(const AcceptParams p) {
  __shared__ double buf0[kMaxFine], buf1[kMaxFine];   // slice sums of the residual and of p
  __shared__ double s_before;
  __shared__ double wave_tot[kThreads / 64];
  __shared__ int s_slice, s_lane, s_last_lane;
  const int nb = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  FoldPair rs;   // requested before the context's own loads, so that both arrive in one round trip
  rs.load(p.rsum + ((size_t)nb * 2 + 0) * p.n_fine, p.rsum + ((size_t)nb * 2 + 1) * p.n_fine, p.n_fine);
  const double u = (double)p.u_sample[nb];
  const ResidCtx<BF16> ctx = make_ctx<BF16>(p, nb);
  // total residual mass; without mass (rounding only) the draw is from p_n itself
  double S, Sp;
  rs.sum(p.n_fine, buf0, buf1, &S, &Sp);
  int mode = 0;
  const double *buf = buf0;
  if (!(S > 0.0)) {   // uniform
    mode = 1;
    S = Sp;
    buf = buf1;
  }
  const double thr = u * S;
  if (wave == 0) {
    // slice in which the running sum (buf still holds the slice sums) first exceeds thr; the last slice with mass
    // if rounding hides the crossing.  Lane j owns `per` consecutive slices; an exclusive scan over the lanes gives
    // the mass before its first one.
    const int per = (p.n_fine + 63) / 64;
    const int c0 = min(p.n_fine, lane * per), c1 = min(p.n_fine, c0 + per);
    double own = 0.0;
    for (int c = c0; c < c1; ++c) own += buf[c];
    double incl = own;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const double up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    const double prev = __shfl_up(incl, 1);
    double acc = lane ? prev : 0.0;
    int cross = INT_MAX, last = -1;
    double before = 0.0, before_last = 0.0;
    for (int c = c0; c < c1; ++c) {
      const double r = buf[c];
      if (r > 0.0) last = c, before_last = acc;
      if (cross == INT_MAX && acc + r > thr) cross = c, before = acc;
      acc += r;
    }
    const uint64_t hit = __ballot(cross != INT_MAX), has = __ballot(last >= 0);
    int cs = 0;
    double bef = 0.0;
    if (hit) {
      const int src = __ffsll((unsigned long long)hit) - 1;
      cs = __shfl(cross, src);
      bef = __shfl(before, src);
    } else if (has) {
      const int src = 63 - __clzll((long long)has);
      cs = __shfl(last, src);
      bef = __shfl(before_last, src);
    }
    if (lane == 0) s_before = bef, s_slice = cs, s_lane = INT_MAX, s_last_lane = -1;
  }
  __syncthreads();
  const int cs = s_slice;
  // lane of that slice whose 8 tokens contain the crossing: inclusive scan of the stored per-lane sums
  const double mine = p.lane_sums[(((size_t)nb * p.n_fine + cs) * kThreads + tid) * 2 + mode];
  double incl = mine;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const double up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  double base = s_before;
  for (int w = 0; w < wave; ++w) base += wave_tot[w];
  const double hi = base + incl, lo = hi - mine;
  if (mine > 0.0) {
    atomicMax(&s_last_lane, tid);
    if (hi > thr && !(lo > thr)) atomicMin(&s_lane, tid);
  }
  __syncthreads();
  const int pick_lane = s_lane != INT_MAX ? s_lane : s_last_lane;
  if (tid == pick_lane) {
    // the lane's eight tokens once more: all loads first, then the eight masses side by side (tokens past V read as
    // -inf and have no mass), then the walk
    const int v0 = cs * kFine + tid * kFinePer;
    const bool vec = ((size_t)p.V * (BF16 ? 2 : 4)) % 16 == 0;
    float tx[kFinePer], dx[kFinePer];
    load_fine<BF16>(ctx.target, ctx.trow, v0, p.V, vec, tx);
    if (ctx.has_draft) load_fine<BF16>(ctx.draft, ctx.drow, v0, p.V, vec, dx);
    double mass[kFinePer];
#pragma unroll
    for (int e = 0; e < kFinePer; ++e) {
      double r, pm;
      ctx.eval(v0 + e, tx[e], ctx.has_draft ? dx[e] : 0.f, r, pm);
      mass[e] = mode ? pm : r;
    }
    double run = lo;
    int tok = -1, last = -1;
#pragma unroll
    for (int e = 0; e < kFinePer; ++e) {
      run += mass[e];
      if (mass[e] > 0.0) {
        last = v0 + e;
        if (tok < 0 && run > thr) tok = v0 + e;
      }
    }
    p.next_token[nb] = tok >= 0 ? tok : last;
  }
}

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

template <bool BF16>
hipError_t launch_typed(const AcceptParams &p, hipStream_t stream) {
  const bool vec = ((size_t)p.V * (BF16 ? 2 : 4)) % 16 == 0;
  {
    ProfileScope scope(SLOT_ACCEPT_STATS, stream);
    const dim3 grid(p.n_chunks, p.draft ? p.NB * (2 * p.K + 1) : p.NB * (p.K + 1));
    if (vec)
      hipLaunchKernelGGL((accept_stats_kernel<BF16, true>), grid, dim3(kThreads), 0, stream, p);
    else
      hipLaunchKernelGGL((accept_stats_kernel<BF16, false>), grid, dim3(kThreads), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (p.warp_key) {
    ProfileScope scope(SLOT_ACCEPT_WARP, stream);
    if (p.top_p < 1.0f && !(p.top_k > 0 && p.top_k < p.V)) {   // top-p alone needs every target row's whole mass
      hipLaunchKernelGGL(accept_rowz_kernel<BF16>, dim3((p.n_fine + kRowzGroup - 1) / kRowzGroup, p.NB * (p.K + 1)),
                         dim3(kThreads), 0, stream, p);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(accept_warp_kernel<BF16>, dim3(p.NB * (p.K + 1)), dim3(kWarpThreads), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  {
    ProfileScope scope(SLOT_ACCEPT_DECIDE, stream);
    hipLaunchKernelGGL(accept_decide_kernel<BF16>, dim3(p.n_fine, p.NB), dim3(kThreads), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  {
    ProfileScope scope(SLOT_ACCEPT_RESID, stream);
    hipLaunchKernelGGL(accept_resid_kernel<BF16>, dim3(p.n_fine, p.NB), dim3(kThreads), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  {
    ProfileScope scope(SLOT_ACCEPT_PICK, stream);
    hipLaunchKernelGGL(accept_pick_kernel<BF16>, dim3(p.NB), dim3(kThreads), 0, stream, p);
    return hipGetLastError();
  }
}

}  // namespace

size_t accept_workspace_bytes(int NB, int K, int V, bool bf16, int *n_chunks_out, int *n_fine_out) {
  const int slice = bf16 ? StatsShape<true>::kSlice : StatsShape<false>::kSlice;
  const int n_chunks = (V + slice - 1) / slice;
  const int n_fine = (V + kFine - 1) / kFine;
  if (n_chunks_out) *n_chunks_out = n_chunks;
  if (n_fine_out) *n_fine_out = n_fine;
  size_t b = 0;
  b += align_up((size_t)NB * (2 * K + 1) * n_chunks * 2 * sizeof(float));  // stats
  b += align_up((size_t)NB * sizeof(int32_t));                             // n_acc
  b += align_up((size_t)NB * 2 * n_fine * sizeof(double));                 // zsum
  b += align_up((size_t)NB * 2 * n_fine * sizeof(double));                 // rsum
  b += align_up((size_t)NB * 2 * sizeof(float));                           // rowmax
  b += align_up((size_t)NB * n_fine * kThreads * 2 * sizeof(double));      // lane_sums
  b += align_up((size_t)NB * (K + 1) * sizeof(uint32_t));                  // warp_key
  b += align_up((size_t)NB * (K + 1) * sizeof(double));                    // warp_z
  b += align_up((size_t)NB * (K + 1) * sizeof(float));                     // warp_max
  b += align_up((size_t)NB * (K + 1) * n_fine * sizeof(double));           // warp_zs
  return b;
}

void accept_carve_workspace(AcceptParams &p, void *ws) {
  uint8_t *at = (uint8_t *)ws;
  p.stats = (float *)at;
  at += align_up((size_t)p.NB * (2 * p.K + 1) * p.n_chunks * 2 * sizeof(float));
  p.n_acc = (int32_t *)at;
  at += align_up((size_t)p.NB * sizeof(int32_t));
  p.zsum = (double *)at;
  at += align_up((size_t)p.NB * 2 * p.n_fine * sizeof(double));
  p.rsum = (double *)at;
  at += align_up((size_t)p.NB * 2 * p.n_fine * sizeof(double));
  p.rowmax = (float *)at;
  at += align_up((size_t)p.NB * 2 * sizeof(float));
  p.lane_sums = (double *)at;
  at += align_up((size_t)p.NB * p.n_fine * kThreads * 2 * sizeof(double));
  const bool warp = (p.top_k > 0 && p.top_k < p.V) || p.top_p < 1.0f;
  p.warp_key = warp ? (uint32_t *)at : nullptr;
  at += align_up((size_t)p.NB * (p.K + 1) * sizeof(uint32_t));
  p.warp_z = warp ? (double *)at : nullptr;
  at += align_up((size_t)p.NB * (p.K + 1) * sizeof(double));
  p.warp_max = warp ? (float *)at : nullptr;
  at += align_up((size_t)p.NB * (p.K + 1) * sizeof(float));
  p.warp_zs = warp ? (double *)at : nullptr;
}

namespace {
__global__ __launch_bounds__(kThreads) void exp64_probe_kernel(const double *y, double *out, size_t n) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < n) out[i] = exp64(y[i]);
}
}  // namespace

hipError_t launch_exp64_probe(const double *y, double *out, size_t n, hipStream_t stream) {
  hipLaunchKernelGGL(exp64_probe_kernel, dim3((unsigned)((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream, y, out,
                     n);
  return hipGetLastError();
}

hipError_t launch_accept(const AcceptParams &p, hipStream_t stream) {
  return p.bf16 ? launch_typed<true>(p, stream) : launch_typed<false>(p, stream);
}

}  // namespace la
