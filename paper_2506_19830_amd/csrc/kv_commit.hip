// KV commit (gfx950): once the verification pass has decided what survives (Algorithm 1: the output
// s^_0 .. s^_{j*-1} (+) s_{j*} is appended to x), the K/V rows of those tokens move from the pass's private
// tensors into the paged prefix cache, for every layer in one launch.
//
// Per request b the appended sequence is  chain[0 .. n_chain)  then  branch[src_branch][0 .. n_own);  token t of it
// lands at position prefix_len + t through the block table.  A thread owns one 16-byte source piece (32 bytes for
// fp32) of one (token, kv head) and moves its K and its V piece, both loads before the stores: reads are contiguous
// over (head, d) of a token, writes are whole rows of the cache.  (More tokens per thread measured slower: the
// launch then has too few wavefronts in flight to cover HBM latency.)  Pure data movement, bound by HBM; with a bf16 source and an fp8 cache the
// piece is quantised on the way: x / scale[head] (fp32 division), clamped to +-448, v_cvt_pk_fp8_f32 (OCP e4m3fn,
// round to nearest even).
#include "la_internal.hpp"

namespace la {
namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

enum CommitMode { COPY_1B = 0, COPY_2B, COPY_4B, QUANT_BF16_FP8 };

__device__ __forceinline__ uint32_t quant4(uint32_t w0, uint32_t w1, float s) {
  // two words of bf16 pairs -> four e4m3 codes in one word, element order kept
  const float x0 = __builtin_bit_cast(float, w0 << 16), x1 = __builtin_bit_cast(float, w0 & 0xffff0000u);
  const float x2 = __builtin_bit_cast(float, w1 << 16), x3 = __builtin_bit_cast(float, w1 & 0xffff0000u);
  auto q = [s](float x) { return __builtin_fminf(__builtin_fmaxf(x / s, -448.0f), 448.0f); };
  uint32_t out = 0;
  out = __builtin_amdgcn_cvt_pk_fp8_f32(q(x0), q(x1), out, false);
  out = __builtin_amdgcn_cvt_pk_fp8_f32(q(x2), q(x3), out, true);
  return out;
}

// Elements per thread and row: 16 bytes of source (fp8: 16 elements) except fp32 (8 elements, 32 bytes).
template <int MODE>
constexpr int kElems = MODE == COPY_1B ? 16 : 8;
constexpr int kTokensPerThread = 1;

template <int MODE>
struct Piece {
  u32x4 a, b;  // b: second half of a 32-byte fp32 piece
};

template <int MODE>
__device__ __forceinline__ Piece<MODE> load_piece(const uint8_t *src, size_t elem) {
  Piece<MODE> r;
  constexpr int es = MODE == COPY_1B ? 1 : MODE == COPY_4B ? 4 : 2;
  r.a = *(const u32x4 *)(src + elem * es);
  if constexpr (MODE == COPY_4B) r.b = *(const u32x4 *)(src + elem * es + 16);
  return r;
}

template <int MODE>
__device__ __forceinline__ void store_piece(uint8_t *dst, size_t elem, const Piece<MODE> &r, float s) {
  if constexpr (MODE == COPY_1B) {
    *(u32x4 *)(dst + elem) = r.a;
  } else if constexpr (MODE == COPY_2B) {
    *(u32x4 *)(dst + elem * 2) = r.a;
  } else if constexpr (MODE == COPY_4B) {
    *(u32x4 *)(dst + elem * 4) = r.a;
    *(u32x4 *)(dst + elem * 4 + 16) = r.b;
  } else {
    u32x2 o = {quant4(r.a[0], r.a[1], s), quant4(r.a[2], r.a[3], s)};
    *(u32x2 *)(dst + elem) = o;
  }
}

template <int MODE>
__global__ __launch_bounds__(256) void kv_commit_kernel(const CommitParams p) {
  const int b = blockIdx.y, layer = blockIdx.z;
  const int src_g = min(max(p.src_branch[b], 0), p.gamma - 1);
  const int n_chain = min(max(p.n_chain[b], 0), p.C);
  const int n_own = min(max(p.n_own[b], 0), p.L);
  const int P = min(max(p.prefix_lens[b], 0), p.capacity);
  const int n_tok = min(n_chain + n_own, p.capacity - P);  // never past what the block table maps
  if (layer == 0 && blockIdx.x == 0 && threadIdx.x == 0) p.new_prefix_lens[b] = P + n_tok;

  const int groups = p.D / kElems<MODE>;  // pieces per row
  const int per_tok = p.Hkv * groups;
  const int item = blockIdx.x * 256 + threadIdx.x;
  const int tq = item / per_tok;  // this thread's tokens: tq*kTokensPerThread ..
  const int t0 = tq * kTokensPerThread;
  if (t0 >= n_tok) return;
  const int rem = item - tq * per_tok;
  const int hk = rem / groups, d0 = (rem - hk * groups) * kElems<MODE>;

  float ks = 1.0f, vs = 1.0f;
  if constexpr (MODE == QUANT_BF16_FP8) {
    if (p.k_scale) ks = p.k_scale[(size_t)layer * p.scale_stride + hk];
    if (p.v_scale) vs = p.v_scale[(size_t)layer * p.scale_stride + hk];
  }
  const uint8_t *kb = (const uint8_t *)p.k_branch, *vb = (const uint8_t *)p.v_branch;
  const uint8_t *kn = (const uint8_t *)p.k_chain, *vn = (const uint8_t *)p.v_chain;

  // all loads of the thread's tokens first, then the stores
  Piece<MODE> kp[kTokensPerThread], vp[kTokensPerThread];
  size_t dst[kTokensPerThread];
#pragma unroll
  for (int j = 0; j < kTokensPerThread; ++j) {
    const int t = min(t0 + j, n_tok - 1);  // surplus slots repeat the last token (and store nothing)
    const int pos = P + t;
    const int lb = pos >> p.block_shift;
    const int blk = p.block_tables ? p.block_tables[(size_t)b * p.max_blocks + lb] : b * p.max_blocks + lb;
    dst[j] = (((size_t)blk * p.Hkv + hk) * p.block_size + (pos & (p.block_size - 1))) * p.D + d0 +
             (size_t)layer * p.cache_stride;
    const bool from_chain = t < n_chain;
    const size_t src = from_chain
                           ? (((size_t)b * p.C + t) * p.Hkv + hk) * p.D + d0 + (size_t)layer * p.chain_stride
                           : ((((size_t)b * p.gamma + src_g) * p.L + (t - n_chain)) * p.Hkv + hk) * p.D + d0 +
                                 (size_t)layer * p.branch_stride;
    kp[j] = load_piece<MODE>(from_chain ? kn : kb, src);
    vp[j] = load_piece<MODE>(from_chain ? vn : vb, src);
  }
#pragma unroll
  for (int j = 0; j < kTokensPerThread; ++j) {
    if (t0 + j < n_tok) {
      store_piece<MODE>((uint8_t *)p.k_cache, dst[j], kp[j], ks);
      store_piece<MODE>((uint8_t *)p.v_cache, dst[j], vp[j], vs);
    }
  }
}

}  // namespace

hipError_t launch_kv_commit(const CommitParams &p, int src_bytes, bool quantise, hipStream_t stream) {
  ProfileScope scope(SLOT_KV_COMMIT, stream);
  const int elems = (!quantise && src_bytes == 1) ? 16 : 8;
  const int items = ((p.C + p.L + kTokensPerThread - 1) / kTokensPerThread) * p.Hkv * (p.D / elems);
  const dim3 grid((items + 255) / 256, p.B, p.num_layers), block(256);
  if (quantise)
    hipLaunchKernelGGL(kv_commit_kernel<QUANT_BF16_FP8>, grid, block, 0, stream, p);
  else if (src_bytes == 1)
    hipLaunchKernelGGL(kv_commit_kernel<COPY_1B>, grid, block, 0, stream, p);
  else if (src_bytes == 2)
    hipLaunchKernelGGL(kv_commit_kernel<COPY_2B>, grid, block, 0, stream, p);
  else if (src_bytes == 4)
    hipLaunchKernelGGL(kv_commit_kernel<COPY_4B>, grid, block, 0, stream, p);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace la
