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

// Tree form: number of pool tokens of request b in [0, lim) whose node is accepted.  Called by every thread of the
// workgroup (contains barriers); 256 tokens per round, one ballot per wavefront.
__device__ __forceinline__ bool pool_token_kept(const CommitParams &p, int b, uint64_t mask, int c) {
  const int seg = p.pool_seg[(size_t)b * p.C + c];
  return seg >= 0 && seg < 64 && ((mask >> seg) & 1u);  // a label outside 0..63 is never kept
}

__device__ int kept_before(const CommitParams &p, int b, uint64_t mask, int lim, int *lds_count) {
  if (threadIdx.x == 0) *lds_count = 0;
  __syncthreads();
  int n = 0;
  for (int base = 0; base < lim; base += 256) {  // uniform trip count: the ballot sees every lane
    const int c = base + threadIdx.x;
    const bool kept = c < lim && pool_token_kept(p, b, mask, c);
    n += __popcll(__ballot(kept));
  }
  if ((threadIdx.x & 63) == 0 && n) atomicAdd(lds_count, n);
  __syncthreads();
  const int total = *lds_count;
  __syncthreads();  // the next call resets the counter
  return total;
}

template <int MODE, bool TREE>
__global__ __launch_bounds__(256) void kv_commit_kernel(const CommitParams p) {
  const int b = blockIdx.y, layer = blockIdx.z;
  const int src_g = min(max(p.src_branch[b], 0), p.gamma - 1);
  const int n_own = min(max(p.n_own[b], 0), p.L);
  const int P = min(max(p.prefix_lens[b], 0), p.capacity);

  const int groups = p.D / kElems<MODE>;  // pieces per row
  const int per_tok = p.Hkv * groups;
  const int item = blockIdx.x * 256 + threadIdx.x;
  const int t0 = item / per_tok;  // this thread's slot: chain / pool token t0, or own token t0 - C

  // t: place of the thread's token in the appended sequence (-1: none); from_chain: it comes from the chain / pool
  int t, n_tok, n_chain = 0;
  bool from_chain;
  if constexpr (TREE) {
    __shared__ int lds_count;
    const uint64_t mask = p.commit_mask[b];
    if (layer == 0 && blockIdx.x == 0) {  // one workgroup per request reports the new length
      const int n_kept = kept_before(p, b, mask, p.C, &lds_count);
      if (threadIdx.x == 0) p.new_prefix_lens[b] = min(P + n_kept + n_own, p.capacity);
    }
    // kept tokens before the workgroup's first slot, then the few between that and the thread's own slot
    const int first = min((blockIdx.x * 256) / per_tok, p.C);
    int rank = kept_before(p, b, mask, first, &lds_count);
    const int upto = min(t0, p.C);
    for (int c = first; c < upto; ++c) rank += pool_token_kept(p, b, mask, c) ? 1 : 0;
    from_chain = t0 < p.C;
    if (from_chain)
      t = pool_token_kept(p, b, mask, t0) ? rank : -1;
    else
      t = t0 - p.C < n_own ? rank + (t0 - p.C) : -1;
    n_tok = p.capacity - P;  // never past what the block table maps
  } else {
    n_chain = p.n_chain ? min(max(p.n_chain[b], 0), p.C) : 0;
    n_tok = min(n_chain + n_own, p.capacity - P);
    if (layer == 0 && blockIdx.x == 0 && threadIdx.x == 0) p.new_prefix_lens[b] = P + n_tok;
    t = t0;
    from_chain = t < n_chain;
  }
  if (t < 0 || t >= n_tok) return;
  const int rem = item - t0 * per_tok;
  const int hk = rem / groups, d0 = (rem - hk * groups) * kElems<MODE>;

  float ks = 1.0f, vs = 1.0f;
  if constexpr (MODE == QUANT_BF16_FP8) {
    if (p.k_scale) ks = p.k_scale[(size_t)layer * p.scale_stride + hk];
    if (p.v_scale) vs = p.v_scale[(size_t)layer * p.scale_stride + hk];
  }
  const uint8_t *kb = (const uint8_t *)p.k_branch, *vb = (const uint8_t *)p.v_branch;
  const uint8_t *kn = (const uint8_t *)p.k_chain, *vn = (const uint8_t *)p.v_chain;

  const int pos = P + t;
  const int lb = pos >> p.block_shift;
  const int blk = p.block_tables ? p.block_tables[(size_t)b * p.max_blocks + lb] : b * p.max_blocks + lb;
  const size_t dst = (((size_t)blk * p.Hkv + hk) * p.block_size + (pos & (p.block_size - 1))) * p.D + d0 +
                     (size_t)layer * p.cache_stride;
  size_t src;
  if constexpr (TREE) {
    src = from_chain ? (((size_t)b * p.C + t0) * p.Hkv + hk) * p.D + d0 + (size_t)layer * p.chain_stride
                     : ((((size_t)b * p.gamma + src_g) * p.L + (t0 - p.C)) * p.Hkv + hk) * p.D + d0 +
                           (size_t)layer * p.branch_stride;
  } else {
    src = from_chain ? (((size_t)b * p.C + t) * p.Hkv + hk) * p.D + d0 + (size_t)layer * p.chain_stride
                     : ((((size_t)b * p.gamma + src_g) * p.L + (t - n_chain)) * p.Hkv + hk) * p.D + d0 +
                           (size_t)layer * p.branch_stride;
  }
  // both loads before the stores
  const Piece<MODE> kp = load_piece<MODE>(from_chain ? kn : kb, src);
  const Piece<MODE> vp = load_piece<MODE>(from_chain ? vn : vb, src);
  store_piece<MODE>((uint8_t *)p.k_cache, dst, kp, ks);
  store_piece<MODE>((uint8_t *)p.v_cache, dst, vp, vs);
}

template <bool TREE>
hipError_t launch(const CommitParams &p, int src_bytes, bool quantise, const dim3 &grid, hipStream_t stream) {
  const dim3 block(256);
  if (quantise)
    hipLaunchKernelGGL((kv_commit_kernel<QUANT_BF16_FP8, TREE>), grid, block, 0, stream, p);
  else if (src_bytes == 1)
    hipLaunchKernelGGL((kv_commit_kernel<COPY_1B, TREE>), grid, block, 0, stream, p);
  else if (src_bytes == 2)
    hipLaunchKernelGGL((kv_commit_kernel<COPY_2B, TREE>), grid, block, 0, stream, p);
  else if (src_bytes == 4)
    hipLaunchKernelGGL((kv_commit_kernel<COPY_4B, TREE>), grid, block, 0, stream, p);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace

hipError_t launch_kv_commit(const CommitParams &p, int src_bytes, bool quantise, hipStream_t stream) {
  ProfileScope scope(SLOT_KV_COMMIT, stream);
  const int elems = (!quantise && src_bytes == 1) ? 16 : 8;
  const int items = (p.C + p.L) * p.Hkv * (p.D / elems);
  const dim3 grid((items + 255) / 256, p.B, p.num_layers);
  return p.pool_seg ? launch<true>(p, src_bytes, quantise, grid, stream)
                    : launch<false>(p, src_bytes, quantise, grid, stream);
}

}  // namespace la
