// Shared-prefix verify attention, streaming shape (gfx950): few query rows per KV head.
//
// With few rows R = gamma*L*G per KV head the pass is bound by the K/V stream of the shared prefix (Algorithm 1:
// every candidate x'_j re-reads x_{1:t}), not by the matrix cores.  This shape is built around keeping that
// stream saturated:
//   * K/V tiles go global -> LDS directly (global_load_lds_dwordx4, 16 bytes per lane, no staging registers), as
//     stored (fp8 stays fp8), NST stages deep, issued NST-1 steps ahead of their use;
//   * the MFMA operands are formed at the fragment read: K rows as they lie (the contraction runs over d) -- with an
//     fp8 cache they feed the fp8 MFMA unconverted, against a two-term fp8 expansion of Q (mfma_kq) --, V through the
//     transposing LDS read (ds_read_b64_tr_b8: each lane receives one head-dim column of eight keys), fp8 widened
//     to bf16 in registers (exact);
//   * a workgroup is eight wavefronts = NRB row blocks of 32 rows x KSL = 8/NRB key slices: per pipeline step of
//     KSL consecutive 64-key tiles, wavefront (rb, ks) reduces tile ks for its 32 rows, so that two wavefronts
//     per SIMD work even when there are only 64 rows; the slices of a row block are folded through LDS at the
//     end and leave one partial per row;
//   * Q comes through LDS as well (fp8 cache: direct loads, each lane fetching exactly what it later reads back,
//     rewritten in place as the fp8 operands while the first K/V tiles are on their way), so that every vector
//     memory operation of the kernel is a direct load whose completion the kernel counts itself;
//   * the unmasked tiles keep the base their probabilities are formed against and never rescale O; they run in a
//     loop of their own, and a workgroup that meets a score far above its base reduces its chunk a second time in a
//     general form (stream_tile_fast says why).
// The last chunk's workgroup also reduces the branch-private keys (causal inside the branch), as further steps
// of the same pipeline.
//
// LDS layout of a tile half (K or V, 64 key rows of 128 bytes): a wavefront-wide load lands as 1 KiB in lane
// order, i.e. eight key rows x eight 16-byte pieces.  Piece p of key k is stored in slot p ^ swz(k); the
// swizzle is applied to the *global* address a lane fetches, and chosen such that the fragment reads
// (16 consecutive keys at one piece for K; eight keys x two pieces for V) spread over all banks.
#include <mutex>
#include <type_traits>

#include "attn_common.hpp"

namespace la {
namespace {

constexpr int kD = 128;
constexpr int kTileN = 64;
constexpr int kRowBytes = kD;                  // fp8
constexpr int kHalfBytes = kTileN * kRowBytes;  // K (or V) part of a tile
constexpr int kTileBytes = 2 * kHalfBytes;      // 16 KiB
constexpr int kMaxBlkLds = 2048;                // block ids of one chunk kept in LDS
constexpr int kWaves = 8;

// Tile geometry by storage type.  A wavefront-wide direct load is 1 KiB: kRows key rows x kPieces 16-byte pieces.
template <bool FP8>
struct Geo {
  static constexpr int kRow = kD * (FP8 ? 1 : 2);     // bytes per key row
  static constexpr int kPieces = kRow / 16;           // 8 / 16
  static constexpr int kRows = 1024 / kRow;           // key rows per load: 8 / 4
  static constexpr int kHalf = kTileN * kRow;         // K (or V) part of a tile: 8 / 16 KiB
  static constexpr int kTile = 2 * kHalf;
  static constexpr int kLoadsPerHalf = kTileN / kRows;  // 8 / 16
};

#define LA_LDS __attribute__((address_space(3)))
typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((ext_vector_type(4))) short i16x4;

// fp8 tiles (8 pieces per row, two rows per 256 bytes of banks)
__device__ __forceinline__ int swz_k(int key) { return (key >> 1) & 7; }
__device__ __forceinline__ int swz_v(int key) { return (((key >> 1) & 1) << 1) | (((key >> 3) & 1) << 2) | ((key >> 2) & 1); }
// bf16 tiles (16 pieces per row = all banks once): one swizzle serves the K reads (16 consecutive keys at one piece
// need 16 different slots) and the transposing V reads (four consecutive keys x an aligned group of four pieces)
__device__ __forceinline__ int swz_16(int key) { return ((key & 3) << 2) | ((key >> 2) & 3); }
template <bool FP8>
__device__ __forceinline__ int swz(int key, int half) {
  return FP8 ? (half ? swz_v(key) : swz_k(key)) : swz_16(key);
}

// s_waitcnt vmcnt(n) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, the other counters left at their maxima)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0070 | 0x0F00);
}

// 16 bytes per lane global -> LDS: the wavefront's 64 pieces land at lds_addr + 16*lane.  Issued from inline
// assembly so that the compiler does not see an LDS write in flight (it would otherwise put a full vmcnt(0) wait
// in front of the transposing LDS reads, which carry no address information for it, and so drain the whole prefetch
// queue in every tile); the kernel orders these loads against its LDS reads itself (wait_vmcnt + s_barrier; the
// barrier is also what keeps the compiler from moving LDS accesses across a pipeline step, so the statement needs
// no memory clobber -- with one, every local whose address a lambda captured would be pinned to scratch memory).
// One wait state lies between the write of M0 and the load that reads it (required on this family for LDS-DMA loads;
// the compiler's hazard handling does not look into an assembly statement).
__device__ __forceinline__ void load_lds16(const void *src, uint32_t lds_addr) {
  lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);  // wavefront-uniform by construction; pin it to a scalar register
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(lds_addr) : "m0");
}

// the same with the address as a wavefront-uniform 64-bit base (scalar registers) plus a 32-bit byte offset per lane
__device__ __forceinline__ void load_lds16(const void *base, uint32_t lane_off, uint32_t lds_addr) {
  lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(lane_off), "s"(base), "s"(lds_addr) : "m0");
}

// eight fp8 (two words) -> eight bf16
__device__ __forceinline__ bf16x8 widen8(uint32_t w0, uint32_t w1) {
  u32x4 v = {fp8x2_to_bf16x2<false>(w0), fp8x2_to_bf16x2<true>(w0), fp8x2_to_bf16x2<false>(w1),
             fp8x2_to_bf16x2<true>(w1)};
  return __builtin_bit_cast(bf16x8, v);
}

// S^T += K Q^T over 64 head dimensions with both operands in fp8 (v_mfma_scale_f32_32x32x64_f8f6f4, e4m3 x e4m3).
// A lane holds 32 bytes per operand: two 16-byte pieces of its key row, and the same head dimensions of its query row.
// The query is a two-term fp8 expansion (hi + lo, see the kernel's first step) carrying a power-of-two block scale:
// the instruction multiplies the products of bytes 0..15 of both lane halves by the scale byte (E8M0) of lane ln, those
// of bytes 16..31 by that of lane 32 + ln; byte U of `qscale` is the lane's scale for head dimensions 64U .. 64U + 63.
typedef __attribute__((ext_vector_type(8))) int i32x8;
template <int U>
__device__ __forceinline__ f32x16 mfma_kq(const i32x8 &k, const i32x8 &q, const f32x16 &c, int qscale) {
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(k, q, c, 0, 0, 0, 127, U, qscale);
}
// two 16-byte LDS reads as one 32-byte operand (formed here, once, so that the operand's eight registers are the ones
// the reads write)
__device__ __forceinline__ i32x8 read_pair(const uint8_t *a, const uint8_t *b) {
  typedef __attribute__((ext_vector_type(4))) int i32x4;
  const i32x4 lo = *(const i32x4 *)a, hi = *(const i32x4 *)b;
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// s_waitcnt vmcnt(later * IPW) for a run-time `later` in 0..MAXL (wavefront-uniform)
template <int IPW, int MAXL>
__device__ __forceinline__ void wait_later(int later) {
  if constexpr (MAXL == 0) {
    wait_vmcnt<0>();
  } else {
    if (later >= MAXL)
      wait_vmcnt<MAXL * IPW>();
    else
      wait_later<IPW, MAXL - 1>(later);
  }
}

// One 64-key tile (fp8, in LDS) against the wavefront's 32 rows, as two 32-key blocks whose MFMA and VALU work
// alternate (S0; S1 next to P0; O += V0 P0 next to P1; O += V1 P1).  Same arithmetic as the row-tile kernel:
// S^T = K Q^T, p = 2^(s - m) with the maximum folded into the accumulator start for unmasked tiles, O^T += V^T P^T.
//   kt        the K half of the tile; the V half lies kHalfBytes on
//   koff[u]   lane's byte offset for piece 2u + lh of key ln (key block 0; block 1 is 32 rows on)
//   voff[db]  lane's byte offset for the transposing read of head-dim block db (first 16 keys; the others 16 rows on)
//   qfrag     the lane's Q operands in LDS, eight 16-byte chunks 1 KiB apart: chunk 4U + 2t + hf = bytes 16hf .. +16
//             of the hi (t = 0) or lo (t = 1) term for head dimensions 64U .. 64U + 63;  qscale: their block scales
template <int MASK>
__device__ __forceinline__ void stream_tile(const uint8_t *kt, const uint8_t *qfrag, int qscale, RowState<1> &st,
                                            const int (&koff)[4], const int (&voff)[4], int lh, int first,
                                            int limit) {
  const uint8_t *vt = kt + kHalfBytes;
  constexpr bool kFastable = MASK == MASK_NONE;
  float binit[1] = {kFastable ? st.base[0] : 0.f};
  auto pv = [&](int kb, const uint32_t (&pb)[1][8]) __attribute__((always_inline)) {
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
      const u32x4 pw = {pb[0][4 * t2], pb[0][4 * t2 + 1], pb[0][4 * t2 + 2], pb[0][4 * t2 + 3]};
      const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
      u32x2 vraw[4];
#pragma unroll
      for (int db = 0; db < 4; ++db)
        vraw[db] = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr8_b64_v2i32((LA_LDS i32x2 *)(
                                                 vt + (kb * 32 + t2 * 16) * kRowBytes + voff[db])));
#pragma unroll
      for (int db = 0; db < 4; ++db)
        st.o[db][0] =
            __builtin_amdgcn_mfma_f32_32x32x16_bf16(widen8(vraw[db][0], vraw[db][1]), pf, st.o[db][0], 0, 0, 0);
    }
  };
  auto exp_offset = [&](float (&off)[1]) __attribute__((always_inline)) {
    off[0] = binit[0] - ((st.m_run[0] == -INFINITY) ? 0.f : st.m_run[0]);
  };

  f32x16 s0[1], s1[1];
  uint32_t p0[1][8], p1[1][8];
  float sum0[1], sum1[1], mt[1], alpha[1], off[1];
  // S^T = K Q^T of both key blocks: per 64 head dimensions one fp8 MFMA with the hi term of Q and one with the lo term,
  // on the two K pieces 4U + lh and 4U + 2 + lh of the lane's key as they lie in LDS.  Unmasked tiles start the
  // accumulators from -base (== the running maximum once one exists), so that the MFMAs deliver s - m and a
  // probability is one exponential.
  {
    const float nb = kFastable ? -st.base[0] : 0.f;
    s0[0] = f32x16{nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb};
    s1[0] = s0[0];
    auto half = [&](auto uc) __attribute__((always_inline)) {
      constexpr int U = decltype(uc)::value;
      const i32x8 qh = read_pair(qfrag + (4 * U) * 1024, qfrag + (4 * U + 1) * 1024);
      const i32x8 ql = read_pair(qfrag + (4 * U + 2) * 1024, qfrag + (4 * U + 3) * 1024);
      const i32x8 ka = read_pair(kt + koff[2 * U], kt + koff[2 * U + 1]);
      const i32x8 kb = read_pair(kt + 32 * kRowBytes + koff[2 * U], kt + 32 * kRowBytes + koff[2 * U + 1]);
      s0[0] = mfma_kq<U>(ka, qh, s0[0], qscale);
      s1[0] = mfma_kq<U>(kb, qh, s1[0], qscale);
      s0[0] = mfma_kq<U>(ka, ql, s0[0], qscale);
      s1[0] = mfma_kq<U>(kb, ql, s1[0], qscale);
    };
    half(std::integral_constant<int, 0>{});
    __builtin_amdgcn_sched_barrier(0);  // (the operands of one half at a time: this form is short of registers, not of time)
    half(std::integral_constant<int, 1>{});
  }
  mask_block<1, MASK>(s0, st, 0, lh, first, limit);
  if constexpr (kFastable) block_probs<1, true>(s0, 1.f, off, p0, sum0);
  block_max<1>(s0, 1.f, binit, mt);
  const bool raise0 = raise_max<1>(mt, st, alpha);
  if (!kFastable || raise0) {
    if (raise0) rescale<1>(st, alpha);
    exp_offset(off);
    block_probs<1, false>(s0, 1.f, off, p0, sum0);
  }
  st.l_run[0] += sum0[0];
  pv(0, p0);
  __builtin_amdgcn_sched_barrier(0);
  mask_block<1, MASK>(s1, st, 1, lh, first, limit);
  if constexpr (kFastable) block_probs<1, true>(s1, 1.f, off, p1, sum1);
  block_max<1>(s1, 1.f, binit, mt);
  const bool raise1 = raise_max<1>(mt, st, alpha);  // the accumulators now hold block 0 in the old units
  if (!kFastable || raise0 || raise1) {  // after a raise in block 0, S1 is no longer relative to the maximum
    if (raise1) rescale<1>(st, alpha);
    exp_offset(off);
    block_probs<1, false>(s1, 1.f, off, p1, sum1);
  }
  if (raise0 || raise1) st.base[0] = (st.m_run[0] == -INFINITY) ? 0.f : st.m_run[0];  // base == running maximum
  st.l_run[0] += sum1[0];
  pv(1, p1);
}

// The same tile once more, written for few registers and little code rather than for speed: one 32-key block after
// the other in a loop that is not unrolled, no block's work overlapped with the other's.  This is the form of the
// second attempt (see stream_tile_fast), which runs almost never; with the faster general form there the kernel would
// need private memory for spilled registers, and a kernel that uses private memory at all streams a tenth slower at
// few rows, whichever path is taken.
template <int MASK>
__device__ __forceinline__ void stream_tile_lean(const uint8_t *kt, const uint8_t *qfrag, int qscale, RowState<1> &st,
                                                 const int (&koff)[4], const int (&voff)[4], int lh, int first,
                                                 int limit) {
  const uint8_t *vt = kt + kHalfBytes;
#pragma clang loop unroll(disable)
  for (int kb = 0; kb < 2; ++kb) {
    const uint8_t *kblk = kt + kb * 32 * kRowBytes;
    f32x16 s[1];
    s[0] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    {
      const i32x8 k0 = read_pair(kblk + koff[0], kblk + koff[1]);
      s[0] = mfma_kq<0>(k0, read_pair(qfrag, qfrag + 1024), s[0], qscale);
      s[0] = mfma_kq<0>(k0, read_pair(qfrag + 2 * 1024, qfrag + 3 * 1024), s[0], qscale);
      const i32x8 k1 = read_pair(kblk + koff[2], kblk + koff[3]);
      s[0] = mfma_kq<1>(k1, read_pair(qfrag + 4 * 1024, qfrag + 5 * 1024), s[0], qscale);
      s[0] = mfma_kq<1>(k1, read_pair(qfrag + 6 * 1024, qfrag + 7 * 1024), s[0], qscale);
    }
    mask_block<1, MASK>(s, st, kb, lh, first, limit);
    const float binit[1] = {0.f};
    float mt[1], alpha[1], off[1], sum[1];
    uint32_t pb[1][8];
    block_max<1>(s, 1.f, binit, mt);
    if (raise_max<1>(mt, st, alpha)) {
      rescale<1>(st, alpha);
      st.base[0] = (st.m_run[0] == -INFINITY) ? 0.f : st.m_run[0];  // base == running maximum
    }
    off[0] = -((st.m_run[0] == -INFINITY) ? 0.f : st.m_run[0]);
    block_probs<1, false>(s, 1.f, off, pb, sum);
    st.l_run[0] += sum[0];
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
      const u32x4 pw = {pb[0][4 * t2], pb[0][4 * t2 + 1], pb[0][4 * t2 + 2], pb[0][4 * t2 + 3]};
      const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const u32x2 vraw = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr8_b64_v2i32((LA_LDS i32x2 *)(
                                                         vt + (kb * 32 + t2 * 16) * kRowBytes + voff[db])));
        st.o[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(widen8(vraw[0], vraw[1]), pf, st.o[db][0], 0, 0, 0);
      }
    }
  }
}

// The unmasked tile again, scheduled by hand: the tile's 24 MFMAs in a fixed order (S^T of block 0: four fp8 MFMAs of
// 64 cycles; S^T of block 1 next to the probabilities of block 0; O += block 0, eight bf16 MFMAs of 32 cycles, next
// to the probabilities of block 1; O += block 1), each preceded by the LDS fragment reads that MFMAs starting up to
// kAheadCycles later need, and followed by the conversions of the next V^T operand, its share of the exponentials,
// and a scheduling fence.  A wavefront issues about one instruction per seven cycles and an LDS read returns after a
// hundred or more, so what the compiler's own order loses is waiting: every fragment must already be on its way
// when the MFMAs before its use are issued.  The probabilities are formed against the base the accumulators were
// started from, and that base is never moved here: this function does not rescale O.  (With code that rescales O
// reachable from the end of its S^T phase, the register allocator keeps O in other registers during the O phases than
// during the S^T phase and the common path pays 64 register copies per tile.)  Probabilities far above 1 are no
// problem for bf16 operands and fp32 sums; what this form cannot do is left to others:
//   * the wavefront's first tile (no base yet; O == 0, l == 0): the base becomes the row maximum over the tile, the
//     probabilities of block 0 are formed again against it and S^T of block 1 is shifted by it;
//   * a row sum above kTrigger = 2^60 (a score 60 log2 units above the first tile's maximum: the fp32 range is not
//     far): the give-up flag of the workgroup is raised, and the kernel reduces the whole chunk again in the general
//     form, which follows the maximum and rescales.  Whatever this form has accumulated by then is discarded.
constexpr float kTrigger = 1152921504606846976.0f;
constexpr int kAheadCycles = 224;
// MFMA m of the tile: 0..7 S^T (block m / 4; head dimensions 64 ((m / 2) % 2) ..; hi or lo term m % 2), 8..23 O.
constexpr int mfma_start(int m) { return m < 8 ? 64 * m : 512 + 32 * (m - 8); }
// fragment reads in the order of their use, and how many of them MFMA m needs:
//   0 hi term of Q, 1 K of block 0, 2 lo term of Q (each two 16-byte reads: head dimensions 0..63);  3, 4, 5 the same
//   for head dimensions 64..127;  6, 7 K of block 1;  8..23 V^T fragments (keys 16 t2 .. +16, head-dim block db; 4 t2 + db)
constexpr int reads_needed(int m) {
  constexpr int upto[8] = {2, 3, 5, 6, 7, 7, 8, 8};
  return m < 8 ? upto[m] : m + 1;
}
constexpr int reads_issued_by(int g) {  // before MFMA g is issued (g = -1: none)
  int n = 0;
  if (g < 0) return 0;
  for (int m = 0; m < 24; ++m)
    if (mfma_start(m) <= mfma_start(g) + kAheadCycles) n = reads_needed(m);
  return n;
}

__device__ __forceinline__ void stream_tile_fast(const uint8_t *kt, const uint8_t *qfrag, int qscale, RowState<1> &st,
                                                 const int (&koff)[4], const int (&voff)[4], int32_t *give_up) {
  // per MFMA: an issue priority that falls with progress through the tile, so that of the two wavefronts of a SIMD
  // the one that is behind wins the arbitration
  auto group_extra = [&](int g) __attribute__((always_inline)) {
    if (g == 0) __builtin_amdgcn_s_setprio(3);
    if (g == 4) __builtin_amdgcn_s_setprio(2);
    if (g == 8) __builtin_amdgcn_s_setprio(1);
    if (g == 16) __builtin_amdgcn_s_setprio(0);
  };
  const uint8_t *vt = kt + kHalfBytes;
  i32x8 q[4];     // 2U + t: hi (t = 0) and lo term for head dimensions 64U ..
  i32x8 kr[2][2];  // block, U: K pieces 4U + lh and 4U + 2 + lh
  u32x2 vr[2][8];
  auto read = [&](int i) __attribute__((always_inline)) {
    if (i < 6) {
      const int U = i / 3, w = i % 3;
      if (w == 0) q[2 * U] = read_pair(qfrag + (4 * U) * 1024, qfrag + (4 * U + 1) * 1024);
      if (w == 1) kr[0][U] = read_pair(kt + koff[2 * U], kt + koff[2 * U + 1]);
      if (w == 2) q[2 * U + 1] = read_pair(qfrag + (4 * U + 2) * 1024, qfrag + (4 * U + 3) * 1024);
    } else if (i < 8) {
      const int U = i - 6;
      kr[1][U] = read_pair(kt + 32 * kRowBytes + koff[2 * U], kt + 32 * kRowBytes + koff[2 * U + 1]);
    } else if (i < 24) {
      const int kb = (i - 8) >> 3, t2 = ((i - 8) >> 2) & 1, db = (i - 8) & 3;
      vr[kb][(i - 8) & 7] = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr8_b64_v2i32((LA_LDS i32x2 *)(
                                                        vt + (kb * 32 + t2 * 16) * kRowBytes + voff[db])));
    }
  };
  auto reads_for = [&](auto gc) __attribute__((always_inline)) {
    constexpr int g = decltype(gc)::value;
#pragma unroll
    for (int i = reads_issued_by(g - 1); i < reads_issued_by(g); ++i) read(i);
  };
  const float nb = -st.base[0];
  const f32x16 c_init = {nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb};
  f32x16 s0[1], s1[1];
  uint32_t p0[1][8], p1[1][8];
  float sum0 = 0.f, sum1 = 0.f;
  auto softmax_share = [&](const f32x16 &sc, int pair, uint32_t (&pc)[8], float &sum) __attribute__((always_inline)) {
    const float e0 = __builtin_amdgcn_exp2f(sc[2 * pair]), e1 = __builtin_amdgcn_exp2f(sc[2 * pair + 1]);
    pc[pair] = pack_bf16(e0, e1);
    sum += e0 + e1;
    asm volatile("" : "+v"(sum), "+v"(pc[pair]));  // here, not wherever the value is first needed
  };
  // S^T MFMA m (0..7)
  auto s_mfma = [&](auto mc) __attribute__((always_inline)) {
    constexpr int m = decltype(mc)::value, kb = m / 4, U = (m / 2) % 2, t = m % 2;
    f32x16 &acc = kb ? s1[0] : s0[0];
    acc = mfma_kq<U>(kr[kb][U], q[2 * U + t], (m % 4) == 0 ? c_init : acc, qscale);
  };
  auto s_group = [&](auto gc) __attribute__((always_inline)) {
    constexpr int g = decltype(gc)::value;
    reads_for(gc);
    s_mfma(gc);
    if constexpr (g >= 4) {  // the probabilities of block 0 beside S^T of block 1
      softmax_share(s0[0], 2 * (g - 4), p0[0], sum0);
      softmax_share(s0[0], 2 * (g - 4) + 1, p0[0], sum0);
    }
    group_extra(g);
    __builtin_amdgcn_sched_barrier(0);
  };
  s_group(std::integral_constant<int, 0>{});
  s_group(std::integral_constant<int, 1>{});
  s_group(std::integral_constant<int, 2>{});
  s_group(std::integral_constant<int, 3>{});
  s_group(std::integral_constant<int, 4>{});
  s_group(std::integral_constant<int, 5>{});
  s_group(std::integral_constant<int, 6>{});
  s_group(std::integral_constant<int, 7>{});
  asm volatile("" : "+v"(s1[0]));  // S^T of block 1 is issued here, not after the branch below
  auto o_group = [&](auto gc, const u32x4 &plo, const u32x4 &phi) __attribute__((always_inline)) {
    constexpr int g = decltype(gc)::value, kb = (g - 8) / 8, u = (g - 8) % 8;
    reads_for(gc);
    st.o[u & 3][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(widen8(vr[kb][u][0], vr[kb][u][1]),
                                                             __builtin_bit_cast(bf16x8, u < 4 ? plo : phi), st.o[u & 3][0],
                                                             0, 0, 0);
    if constexpr (kb == 0) softmax_share(s1[0], u, p1[0], sum1);  // the probabilities of block 1 beside O += block 0
    group_extra(g);
    __builtin_amdgcn_sched_barrier(0);
  };
  if (__builtin_expect(__builtin_amdgcn_ballot_w64(st.m_run[0] == -INFINITY) != 0, 0)) {  // (all lanes or none)
    float m = fmaxf(s0[0][0], s1[0][0]);  // (the base is still 0: these are the scores themselves)
#pragma unroll
    for (int j = 1; j < 16; ++j) m = fmaxf(m, fmaxf(s0[0][j], s1[0][j]));
    m = xhalf_max(m);
    st.m_run[0] = m, st.base[0] = m;
    const float off[1] = {-m};
    float sum[1];
    block_probs<1, false>(s0, 1.f, off, p0, sum);
    sum0 = sum[0];
#pragma unroll
    for (int j = 0; j < 16; ++j) s1[0][j] -= m;
  }
  if (!(sum0 <= kTrigger)) *(volatile int32_t *)give_up = 1;
  st.l_run[0] += sum0;
  const u32x4 pa0 = {p0[0][0], p0[0][1], p0[0][2], p0[0][3]}, pa1 = {p0[0][4], p0[0][5], p0[0][6], p0[0][7]};
  o_group(std::integral_constant<int, 8>{}, pa0, pa1);
  o_group(std::integral_constant<int, 9>{}, pa0, pa1);
  o_group(std::integral_constant<int, 10>{}, pa0, pa1);
  o_group(std::integral_constant<int, 11>{}, pa0, pa1);
  o_group(std::integral_constant<int, 12>{}, pa0, pa1);
  o_group(std::integral_constant<int, 13>{}, pa0, pa1);
  o_group(std::integral_constant<int, 14>{}, pa0, pa1);
  o_group(std::integral_constant<int, 15>{}, pa0, pa1);
  if (!(sum1 <= kTrigger)) *(volatile int32_t *)give_up = 1;
  st.l_run[0] += sum1;
  const u32x4 pb0 = {p1[0][0], p1[0][1], p1[0][2], p1[0][3]}, pb1 = {p1[0][4], p1[0][5], p1[0][6], p1[0][7]};
  o_group(std::integral_constant<int, 16>{}, pb0, pb1);
  o_group(std::integral_constant<int, 17>{}, pb0, pb1);
  o_group(std::integral_constant<int, 18>{}, pb0, pb1);
  o_group(std::integral_constant<int, 19>{}, pb0, pb1);
  o_group(std::integral_constant<int, 20>{}, pb0, pb1);
  o_group(std::integral_constant<int, 21>{}, pb0, pb1);
  o_group(std::integral_constant<int, 22>{}, pb0, pb1);
  o_group(std::integral_constant<int, 23>{}, pb0, pb1);
  __builtin_amdgcn_s_setprio(0);
}

// The direct K/V loads of one wavefront.  A step is KSL tiles x (8 + 8) loads of 1 KiB (eight key rows each);
// wavefront w issues loads w*IPW .. w*IPW + IPW-1 of every step.  Lane l fetches 16 bytes of key row l/8 of those
// eight: slot l%8, i.e. global piece (l%8) ^ swz(key).  Every wavefront issues exactly IPW loads per step, so the
// load counter advances uniformly; where a step reaches past the end of its key range (a ragged last tile, a tile
// slot that has no tile) the tokens are clamped to the last valid one and all addresses stay in bounds.
// (A plain struct of values rather than a capturing lambda: captured locals would be pinned to scratch memory.)
// SBASE: full prefix steps by issue_full_prefix (the second attempt does without: less code)
template <int KSL, int NST, int IPW, bool FP8 = true, bool SBASE = true>
struct StreamLoader {
  using G = Geo<FP8>;
  uint32_t ring;                 // LDS address of the ring
  int wave;
  const int32_t *blk;            // LDS: block ids of the chunk (paged), or null: block = ident + logical block
  int first_lb, ident, shift, bs_mask;
  uint32_t blk_stride, br_stride;  // bytes between cache blocks / between branch tokens
  const uint8_t *k_pre, *v_pre, *k_br, *v_br;
  int key[IPW], goff[IPW];       // per lane: key inside the tile, byte offset inside the key row
  const int32_t *table;          // global: the request's block table (paged), or null
  uint32_t row_off;              // per lane: byte offset of its key row inside the G::kRows rows of a load

  __device__ __forceinline__ void init_lane(int lane) {
#pragma unroll
    for (int j = 0; j < IPW; ++j) {
      const int ii = wave * IPW + j;
      const int half = (ii / G::kLoadsPerHalf) & 1, r = ii % G::kLoadsPerHalf;
      const int k = G::kRows * r + lane / G::kPieces;
      key[j] = k;
      goff[j] = ((lane % G::kPieces) ^ swz<FP8>(k, half)) * 16;
    }
    row_off = (uint32_t)(lane / G::kPieces) * G::kRow;
  }
  // Load j of a step all of whose keys are prefix keys.  The G::kRows key rows of a load start at a multiple of
  // G::kRows tokens and a cache block holds a multiple of 16, so they lie in one block: block id and address base are
  // wavefront-uniform and are formed by the scalar unit (the block id by a scalar load from the table), which leaves
  // the vector ALU -- what the tile's conversions are bound by -- one addition per load.
  __device__ __forceinline__ void issue_full_prefix(int j, int slot, int first0) const {
    typedef const __attribute__((address_space(4))) int32_t *cint_ptr;
    const int ii = wave * IPW + j;
    const int tile = ii / (2 * G::kLoadsPerHalf), half = (ii / G::kLoadsPerHalf) & 1, r = ii % G::kLoadsPerHalf;
    const int tok0 = __builtin_amdgcn_readfirstlane(first0 + tile * kTileN + G::kRows * r);
    const int lb = tok0 >> shift;
    const uint32_t b = table ? (uint32_t)((cint_ptr)(uintptr_t)table)[lb] : (uint32_t)(ident + lb);
    const uint8_t *base = (half ? v_pre : k_pre) + ((uint64_t)b * blk_stride + (uint32_t)(tok0 & bs_mask) * G::kRow);
    load_lds16(base, row_off + (uint32_t)goff[j], ring + slot * (KSL * G::kTile) + tile * G::kTile + half * G::kHalf + r * 1024);
  }
  // PREFIX: cache tokens first0 .. (through the block table); else branch tokens.  CLAMP: tokens above `last`
  // repeat token `last`.
  template <bool PREFIX, bool CLAMP>
  __device__ __forceinline__ void issue(int slot, int first0, int last) const {
#pragma unroll
    for (int j = 0; j < IPW; ++j) {
      if constexpr (PREFIX && !CLAMP && SBASE)
        issue_full_prefix(j, slot, first0);
      else
        issue_one<PREFIX, CLAMP>(j, slot, first0, last);
    }
  }
  // load j (0 .. IPW-1) of a step in the general form (per-lane addresses: clamped tokens, branch tokens)
  template <bool PREFIX, bool CLAMP>
  __device__ __forceinline__ void issue_one(int j, int slot, int first0, int last) const {
    const uint32_t stage = ring + slot * (KSL * G::kTile);
    {
      const int ii = wave * IPW + j;  // wavefront-uniform: which 1 KiB of the step
      const int tile = ii / (2 * G::kLoadsPerHalf), half = (ii / G::kLoadsPerHalf) & 1, r = ii % G::kLoadsPerHalf;
      int tok = first0 + tile * kTileN + key[j];
      if (CLAMP) tok = min(tok, last);
      const uint8_t *src;
      if (PREFIX) {
        const int lb = tok >> shift;
        const uint32_t b = blk ? (uint32_t)blk[lb - first_lb] : (uint32_t)(ident + lb);
        const uint32_t inner = (uint32_t)(tok & bs_mask) * G::kRow + (uint32_t)goff[j];
        src = (half ? v_pre : k_pre) + ((uint64_t)b * blk_stride + inner);  // one 32 x 32 + 64 multiply-add
      } else {
        src = (half ? v_br : k_br) + ((uint64_t)(uint32_t)tok * br_stride + (uint32_t)goff[j]);
      }
      load_lds16(src, stage + tile * G::kTile + half * G::kHalf + r * 1024);
    }
  }
};

// NRB row blocks of 32 rows per workgroup; KSL = 8/NRB tiles per pipeline step; a ring of kSlots tile slots behind
// the Q fragments.
template <int NRB>
struct StreamShape {
  static constexpr int KSL = kWaves / NRB;
  static constexpr int kScaleOff = NRB * 8192;       // behind Q of the row blocks (MFMA operands): their block scales,
  static constexpr int kFlagOff = kScaleOff + NRB * 512;  // [row block][U][lane] words; then the give-up flag
  static constexpr int kQBytes = kScaleOff + (NRB * 512 + 16 + 1023) / 1024 * 1024;
  static constexpr int kRingOff = kQBytes;
  static constexpr int kSlots = ((152 * 1024 - kQBytes) / kTileBytes) / KSL * KSL;
  static constexpr int NST = kSlots / KSL;           // steps the ring holds
  static constexpr int IPW = 16 * KSL / kWaves;      // direct loads per wavefront and step
  static constexpr int kBlkOff = kRingOff + kSlots * kTileBytes;
  static constexpr int kLdsMax = kBlkOff + kMaxBlkLds * 4;
  static_assert(NST >= 2, "one step in flight while another is computed on");
  static_assert(kLdsMax <= 160 * 1024, "LDS of one CU");
  static constexpr int kFoldBytes = kWaves * 66 * 64 * 4;  // the fold of the key slices reuses the whole space
  static_assert(kFoldBytes <= kLdsMax, "fold space");
};

// The work of one workgroup.  GENERAL: every tile in the general form (the second attempt; see stream_tile_fast).
// Returns false if this attempt gave up (nothing has been written then).
template <int NRB, bool GENERAL>
__device__ __forceinline__ bool stream_chunk(const AttnParams &p, uint8_t *lds, int thread_id, int block_id) {
  using S = StreamShape<NRB>;
  constexpr int KSL = S::KSL, NST = S::NST, IPW = S::IPW;
  constexpr int NT = 64 * kWaves;
  constexpr int kTileM = 32 * NRB;
  constexpr int kStepBytes = KSL * kTileBytes;
  const int tid = thread_id;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ln = lane & 31, lh = lane >> 5;
  const int rb = wave % NRB, ks = wave / NRB;

  // ---- which (kv head, row tile, request, chunk) -------------------------------------------
  // (integer divisions run in vector registers; pinning the results to scalar registers keeps what depends on
  // them -- the scale loads among it -- on the scalar side, away from the vector memory counter)
  int id = block_id;
  const int kvh = __builtin_amdgcn_readfirstlane(id % p.Hkv);
  id = __builtin_amdgcn_readfirstlane(id / p.Hkv);
  const int row_tile = __builtin_amdgcn_readfirstlane(id % p.n_row_tiles);
  int c = __builtin_amdgcn_readfirstlane(id / p.n_row_tiles);
  const ChunkSel sel = attn_select_chunk(p, c);
  const int b = sel.b, n_chunks = sel.n_chunks, k_begin = sel.k_begin, k_end = sel.k_end;
  c = sel.c;
  const int n_pre_tiles = (k_end - k_begin + kTileN - 1) / kTileN;
  const int n_pre_steps = (n_pre_tiles + KSL - 1) / KSL;
  const int n_full_steps = (k_end - k_begin) / (KSL * kTileN);  // steps all of whose keys exist

  const int r0 = row_tile * kTileM;
  const int r1 = min(p.R, r0 + kTileM);
  const int gl = p.gamma * p.L;
  // (integer divisions run in vector registers; these values are the same in every lane)
  const int t_lo = __builtin_amdgcn_readfirstlane(r0 / p.G), t_hi = __builtin_amdgcn_readfirstlane((r1 - 1) / p.G);
  const int tk0 = __builtin_amdgcn_readfirstlane((t_lo / p.L) * p.L);
  const int n_priv = (c == n_chunks - 1) ? (t_hi - tk0 + 1 + kTileN - 1) / kTileN : 0;
  const int n_steps = n_pre_steps + (n_priv + KSL - 1) / KSL;

  // ---- physical block ids of this chunk -> LDS (paged caches only) ------------------------------
  int32_t *blk_lds = (int32_t *)(lds + S::kBlkOff);
  const int first_lb = k_begin >> p.block_shift;
  const int32_t *table = p.block_tables ? p.block_tables + (size_t)b * p.max_blocks : nullptr;
  if (table) {  // (uniform over the workgroup)
    if (k_end > k_begin) {
      const int n_blk = ((k_end - 1) >> p.block_shift) - first_lb + 1;  // <= kMaxBlkLds (host guarantees)
      for (int i = tid; i < n_blk; i += NT) blk_lds[i] = table[first_lb + i];
    }
    __syncthreads();
  }
  const uint32_t lds0 = (uint32_t)(size_t)(LA_LDS uint8_t *)lds;
  int32_t *give_up = (int32_t *)(lds + S::kFlagOff);
  if (tid == 0) *give_up = GENERAL ? 0 : p.force_again;  // (published by the barriers of the Q rewrite below)

  // ---- Q -> LDS: wavefront rb < NRB fetches the fragments of row block rb, lane (ln, lh) exactly the 16 bytes
  //      of its row that it (and the same lane of every wavefront of that row block) reads back for MFMA step s:
  //      d = 32*(s/2) + 16*lh + 8*(s%2) .. +8, the halves of the K piece the lane reads.  Rows past R repeat
  //      row R-1 (their fragments are zeroed after the read-back).
  const int row = r0 + rb * 32 + ln;
  const int rr = min(row, p.R - 1);
  const int row_tok = rr / p.G;
  if (wave < NRB) {
    const uint8_t *qrow = (const uint8_t *)p.q + (((size_t)b * gl + row_tok) * p.Hq + kvh * p.G + (rr % p.G)) * (size_t)(kD * 2);
#pragma unroll
    for (int s = 0; s < 8; ++s)
      load_lds16(qrow + (32 * (s >> 1) + 16 * lh + 8 * (s & 1)) * 2, lds0 + wave * 8192 + s * 1024);
  }

  // ---- the direct K/V loads of this wavefront; the stream starts now ----------------------------------
  const size_t br_off = ((size_t)b * gl * p.Hkv + kvh) * kRowBytes;
  StreamLoader<KSL, NST, IPW, true, !GENERAL> ld;
  ld.ring = lds0 + S::kRingOff, ld.wave = wave;
  ld.blk = table ? blk_lds : nullptr, ld.table = table;
  ld.first_lb = first_lb, ld.ident = b * p.max_blocks, ld.shift = p.block_shift, ld.bs_mask = p.block_size - 1;
  ld.blk_stride = (uint32_t)((p.Hkv << p.block_shift) * kRowBytes), ld.br_stride = (uint32_t)(p.Hkv * kRowBytes);
  ld.k_pre = (const uint8_t *)p.k_cache + ((size_t)kvh << p.block_shift) * kRowBytes;
  ld.v_pre = (const uint8_t *)p.v_cache + ((size_t)kvh << p.block_shift) * kRowBytes;
  ld.k_br = (const uint8_t *)p.k_branch + br_off;
  ld.v_br = (const uint8_t *)p.v_branch + br_off;
  ld.init_lane(lane);
  auto issue = [&](int step) __attribute__((always_inline)) {
    const int slot = step % NST;
    if (step < n_full_steps)
      ld.template issue<true, false>(slot, k_begin + step * (KSL * kTileN), 0);
    else if (step < n_pre_steps)
      ld.template issue<true, true>(slot, k_begin + step * (KSL * kTileN), k_end - 1);
    else
      ld.template issue<false, true>(slot, tk0 + (step - n_pre_steps) * (KSL * kTileN), t_hi);
  };
  for (int s = 0; s < NST - 1; ++s)
    if (s < n_steps) issue(s);

  // ---- scales, fragment read offsets ---------------------------------------------------------------
  float c_prefix = p.scale_log2;
  float v_out = 1.0f;
  {
    // read through the constant address space: a wavefront-uniform load from there is a scalar load, which the
    // vector memory counter (the direct loads in flight) does not see
    typedef const __attribute__((address_space(4))) float *cfloat_ptr;
    const float ksc = p.k_scale ? ((cfloat_ptr)(uintptr_t)p.k_scale)[kvh] : 1.0f;
    const float vsc = p.v_scale ? ((cfloat_ptr)(uintptr_t)p.v_scale)[kvh] : 1.0f;
    c_prefix *= ksc;
    v_out = vsc;
  }
  int koff[4], voff[4];
  {
    const int fk = swz_k(ln);  // keys ln and 32 + ln share the swizzle
#pragma unroll
    for (int u = 0; u < 4; ++u) koff[u] = ln * kRowBytes + (((2 * u + lh) ^ fk) * 16);
    // transposing read: the 16 lanes of a group address eight keys x two 8-byte halves of one 16-byte piece; lane i
    // of the group then holds column i of those eight keys
    const int grp = lane >> 4, a = lane & 15, j = a >> 1;
    const int keyl = 8 * (j >> 2) + 4 * (grp >> 1) + (j & 3);
    const int fv = swz_v(keyl);  // the same for the key groups 16, 32, 48 rows on
#pragma unroll
    for (int db = 0; db < 4; ++db) voff[db] = keyl * kRowBytes + (((2 * db + (grp & 1)) ^ fv) * 16) + 8 * (a & 1);
  }
  RowState<1> st;
  st.row_tok[0] = row_tok;
  st.row_bstart[0] = (row_tok / p.L) * p.L;
  st.m_run[0] = -INFINITY;
  st.l_run[0] = 0.f;
  st.base[0] = 0.f;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int j = 0; j < 16; ++j) st.o[db][0][j] = 0.f;

  // ---- Q as the fp8 MFMA's operand ------------------------------------------------------------------------
  int qscale;
  {
    // Q was requested before any K/V, and loads complete in order: it has landed once no more loads are outstanding
    // than the K/V loads issued since.
    wait_later<IPW, NST - 1>(min(NST - 1, n_steps));
    __syncthreads();
    // Multiply by the prefix score scale (log2 units, k_scale folded in) and rewrite it as the fp8 MFMA's operand: per
    // block of 32 head dimensions of a row (16 in this lane, 16 in the lane 32 on) a power-of-two scale 2^E that
    // brings the block's largest magnitude into [128, 256), then x = q' 2^-E = hi + lo + (an error below 2^-8 |x|),
    // hi = fp8(x), lo = fp8(x - hi) -- as good as the bf16 rounding it replaces.  Each key slice of the row block
    // converts a share of the blocks: all read, then (barrier) all write, since the new layout overlaps the old
    // one; one more barrier publishes it.  All of this runs while the first K/V tiles are still on their way.
    constexpr int kNB = 4 / KSL;  // blocks per wavefront; block bi = 2U + hf is fragments 2bi, 2bi + 1
    u32x4 hi[kNB], lo[kNB];
    int ebyte[kNB];
#pragma unroll
    for (int i = 0; i < kNB; ++i) {
      const int bi = ks * kNB + i;
      const uint8_t *at = lds + rb * 8192 + (2 * bi) * 1024 + lane * 16;
      u32x4 va = *(const u32x4 *)at, vb = *(const u32x4 *)(at + 1024);
      if (row >= p.R) va = vb = u32x4{0, 0, 0, 0};
      float x[16];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        x[2 * w] = __builtin_bit_cast(float, va[w] << 16) * c_prefix;
        x[2 * w + 1] = __builtin_bit_cast(float, va[w] & 0xffff0000u) * c_prefix;
        x[8 + 2 * w] = __builtin_bit_cast(float, vb[w] << 16) * c_prefix;
        x[8 + 2 * w + 1] = __builtin_bit_cast(float, vb[w] & 0xffff0000u) * c_prefix;
      }
      float mx = 0.f;
#pragma unroll
      for (int j = 0; j < 16; ++j) mx = fmaxf(mx, fabsf(x[j]));
      mx = xhalf_max(mx);
      int e = (int)((__builtin_bit_cast(uint32_t, mx) >> 23) & 255u) - 127 - 7;
      e = mx > 0.f ? max(-100, min(100, e)) : 0;
      ebyte[i] = 127 + e;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float x0 = __builtin_ldexpf(x[4 * w], -e), x1 = __builtin_ldexpf(x[4 * w + 1], -e);
        const float x2 = __builtin_ldexpf(x[4 * w + 2], -e), x3 = __builtin_ldexpf(x[4 * w + 3], -e);
        int hw = __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, 0, false);
        hw = __builtin_amdgcn_cvt_pk_fp8_f32(x2, x3, hw, true);
        const f32x2 b0 = __builtin_amdgcn_cvt_pk_f32_fp8(hw, false), b1 = __builtin_amdgcn_cvt_pk_f32_fp8(hw, true);
        int lw = __builtin_amdgcn_cvt_pk_fp8_f32(x0 - b0[0], x1 - b0[1], 0, false);
        lw = __builtin_amdgcn_cvt_pk_fp8_f32(x2 - b1[0], x3 - b1[1], lw, true);
        hi[i][w] = (uint32_t)hw, lo[i][w] = (uint32_t)lw;
      }
      __builtin_amdgcn_sched_barrier(0);  // one block at a time (up to four: their temporaries would not fit together)
    }
    __syncthreads();
    int32_t *sc = (int32_t *)(lds + S::kScaleOff) + rb * 128;
#pragma unroll
    for (int i = 0; i < kNB; ++i) {
      const int bi = ks * kNB + i, U = bi >> 1, hf = bi & 1;
      uint8_t *to = lds + rb * 8192 + (4 * U + hf) * 1024 + lane * 16;
      *(u32x4 *)to = hi[i];
      *(u32x4 *)(to + 2048) = lo[i];
      if (lh == 0) sc[U * 64 + hf * 32 + ln] = ebyte[i];
    }
    __syncthreads();
    qscale = sc[lane] | (sc[64 + lane] << 8);
  }

  // ---- the pipeline -------------------------------------------------------------------------------
  const bool active = r0 + rb * 32 < p.R;
  const uint8_t *qfrag = lds + rb * 8192 + lane * 16;
  int step = 0;
  // The steps all of whose tiles are full prefix tiles, in a loop of their own that holds nothing but the
  // hand-scheduled tile: with a tile form that rescales O inside the same loop (the ragged last tile, the
  // branch-private tiles) the register allocator settles O's place at the loop's end by what those forms leave,
  // and the hand-scheduled tile pays 32 register copies per trip to get there.
  if constexpr (!GENERAL) {
    for (; step < n_full_steps; ++step) {
      wait_later<IPW, NST - 2>(min(n_steps - 1, step + NST - 2) - step);
      __builtin_amdgcn_s_barrier();
      if (step + NST - 1 < n_steps) issue(step + NST - 1);
      if (active)
        stream_tile_fast(lds + S::kRingOff + (step % NST) * kStepBytes + ks * kTileBytes, qfrag, qscale, st, koff, voff,
                         give_up);
    }
  }
  for (; step < n_steps; ++step) {
    // own loads of this step have landed (the steps issued after it may still be in flight) ...
    wait_later<IPW, NST - 2>(min(n_steps - 1, step + NST - 2) - step);
    __builtin_amdgcn_s_barrier();  // ... and so have everyone else's; the slots read in the previous step are free
    // the loads of step + NST - 1, in one run: for a full prefix step they are scalar work (issue_full_prefix)
    if (step + NST - 1 < n_steps) issue(step + NST - 1);
    if (!active) continue;
    const uint8_t *kt = lds + S::kRingOff + (step % NST) * kStepBytes + ks * kTileBytes;
    if (step < n_pre_steps) {
      const int first = k_begin + (step * KSL + ks) * kTileN;
      if constexpr (GENERAL) {
        if (first < k_end) stream_tile_lean<MASK_TAIL>(kt, qfrag, qscale, st, koff, voff, lh, first, k_end);
      } else {
        if (first + kTileN <= k_end)
          stream_tile_fast(kt, qfrag, qscale, st, koff, voff, give_up);
        else if (first < k_end)
          stream_tile<MASK_TAIL>(kt, qfrag, qscale, st, koff, voff, lh, first, k_end);
      }
    } else {
      const int first = tk0 + ((step - n_pre_steps) * KSL + ks) * kTileN;
      if (first <= t_hi) {
        if constexpr (GENERAL)
          stream_tile_lean<MASK_BRANCH>(kt, qfrag, qscale, st, koff, voff, lh, first, 0);
        else
          stream_tile<MASK_BRANCH>(kt, qfrag, qscale, st, koff, voff, lh, first, 0);
      }
    }
  }
  wait_vmcnt<0>();  // no direct load may still be on its way to LDS when the workgroup gives its LDS back
  if constexpr (!GENERAL) {
    __syncthreads();  // every wavefront's flag store has landed (the fence waits for it) before anyone reads the flag
    if (__builtin_expect(*(volatile int32_t *)give_up != 0, 0)) return false;
  }

  // ---- fold the key slices of a row block through LDS, every wavefront a share of the columns ----------------
  // All 8/NRB slices of a row block leave (O, m, l) per lane in LDS, layout [wavefront][value 0..65][lane];
  // wavefront `slice` of the row block then combines accumulator registers slice*kPer .. +kPer of all slices and
  // writes those columns of the partial.  Register i = 16*db + j of a lane is head-dim column
  // 32*db + 8*(j/4) + 4*lh + j%4 of its row.
  constexpr int kSlices = kWaves / NRB, kPer = 64 / kSlices;
  const size_t slot = (size_t)b * p.s_max + c;
  const size_t out_row = slot * p.n_rows + (size_t)row_tok * p.Hq + kvh * p.G + (row % p.G);
  float *po = p.part_o + out_row * kD;
  if constexpr (kSlices == 1) {  // one slice: the registers are the partial
    const float l_tot = xhalf_sum(st.l_run[0]);
    if (row < p.R) {
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 v = {st.o[db][0][4 * q] * v_out, st.o[db][0][4 * q + 1] * v_out,
                           st.o[db][0][4 * q + 2] * v_out, st.o[db][0][4 * q + 3] * v_out};
          *(f32x4 *)(po + 32 * db + 8 * q + 4 * lh) = v;
        }
      if (lh == 0) {
        const f32x2 ml = {st.m_run[0], l_tot};
        *(f32x2 *)(p.part_ml + out_row * 2) = ml;
      }
    }
  } else {
    __builtin_amdgcn_s_barrier();  // every wavefront is done with the ring
    float *fold = (float *)lds;
    {
      float *dst = fold + (size_t)wave * 66 * 64 + lane;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int j = 0; j < 16; ++j) dst[(db * 16 + j) * 64] = st.o[db][0][j];
      dst[64 * 64] = st.m_run[0];
      dst[65 * 64] = st.l_run[0];
    }
    __syncthreads();
    const int slice = ks;
    float w[kSlices], m_all = -INFINITY, l_all = 0.f;
#pragma unroll
    for (int s = 0; s < kSlices; ++s) {
      w[s] = fold[(size_t)(s * NRB + rb) * 66 * 64 + 64 * 64 + lane];
      m_all = fmaxf(m_all, w[s]);
    }
    const float m_use = (m_all == -INFINITY) ? 0.f : m_all;
#pragma unroll
    for (int s = 0; s < kSlices; ++s) {
      w[s] = __builtin_amdgcn_exp2f(w[s] - m_use);  // 0 for a slice that saw no key
      l_all = __builtin_fmaf(w[s], fold[(size_t)(s * NRB + rb) * 66 * 64 + 65 * 64 + lane], l_all);
    }
    float acc[kPer];
#pragma unroll
    for (int i = 0; i < kPer; ++i) acc[i] = 0.f;
#pragma unroll
    for (int s = 0; s < kSlices; ++s) {
      const float *src = fold + ((size_t)(s * NRB + rb) * 66 + slice * kPer) * 64 + lane;
#pragma unroll
      for (int i = 0; i < kPer; ++i) acc[i] = __builtin_fmaf(w[s], src[i * 64], acc[i]);
    }
    const float l_tot = xhalf_sum(l_all);
    if (row < p.R) {
#pragma unroll
      for (int i = 0; i < kPer; i += 4) {
        const int reg = slice * kPer + i;  // (wavefront-uniform)
        const f32x4 v = {acc[i] * v_out, acc[i + 1] * v_out, acc[i + 2] * v_out, acc[i + 3] * v_out};
        *(f32x4 *)(po + 32 * (reg >> 4) + 8 * ((reg & 15) >> 2) + 4 * lh) = v;
      }
      if (slice == 0 && lh == 0) {
        const f32x2 ml = {m_all, l_tot};
        *(f32x2 *)(p.part_ml + out_row * 2) = ml;
      }
    }
  }
  return true;
}

template <int NRB>
__global__ __launch_bounds__(64 * kWaves) void attn_stream_kernel(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  if (__builtin_expect(!stream_chunk<NRB, false>(p, lds, threadIdx.x, blockIdx.x), 0)) {
    // The second attempt starts from the kernel's arguments again, and from thread and workgroup ids the compiler
    // cannot see through: whatever it shared between the two attempts stayed alive across the first one, in private
    // memory (a kernel that uses private memory at all streams a tenth slower at few rows).
    int thread_id = threadIdx.x, block_id = blockIdx.x;
    asm volatile("" : "+v"(thread_id), "+s"(block_id));
    stream_chunk<NRB, true>(p, lds, thread_id, block_id);
  }
}

// ---------------------------------------------------------------------------------------------------------------
// bf16 cache and branch K/V: the same pipeline without any conversion.  K fragments are 16-byte LDS reads (the
// contraction runs over d, MFMA step t takes d = 16t + 8lh .. +8 of key ln), V^T fragments two transposing reads
// (ds_read_b64_tr_b16: four keys of one head-dim column each).  Used with many rows per KV head (256-row or
// 128-row workgroups), where it replaces the register-staged row-tile kernel: no staging instructions at all, no
// vector memory wait inside the loop.  Q lives in registers (loaded before the stream starts).
//   koff0         lane's byte offset for piece lh of key ln (key block 0; block 1 is 32 rows on)
//   voff[a][db]   lane's byte offset for the transposing read of keys 8a + 4lh .. +4 of head-dim block db (key group 0
//                 of key block 0; the others 16 / 32 rows on)
// KEEP (unmasked tiles only): the base is never moved and O never rescaled, as in stream_tile_fast and for its
// reason; `give_up` is the workgroup's flag.
template <int MASK, bool KEEP = false>
__device__ __forceinline__ void stream_tile16(const uint8_t *kt, RowState<1> &st, int koff0,
                                              const int (&voff)[2][4], int lh, int first, int limit,
                                              int32_t *give_up = nullptr) {
  static_assert(!KEEP || MASK == MASK_NONE, "only unmasked tiles keep their base");
  using G = Geo<false>;
  const uint8_t *vt = kt + G::kHalf;
  constexpr bool kFastable = MASK == MASK_NONE;
  float binit[1] = {kFastable ? st.base[0] : 0.f};
  auto pv = [&](int kb, const uint32_t (&pb)[1][8]) __attribute__((always_inline)) {
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
      const u32x4 pw = {pb[0][4 * t2], pb[0][4 * t2 + 1], pb[0][4 * t2 + 2], pb[0][4 * t2 + 3]};
      const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
      u32x2 lo[4], hi[4];
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const uint8_t *at = vt + (kb * 32 + t2 * 16) * G::kRow;
        lo[db] = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((LA_LDS i16x4 *)(at + voff[0][db])));
        hi[db] = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((LA_LDS i16x4 *)(at + voff[1][db])));
      }
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const u32x4 vw = {lo[db][0], lo[db][1], hi[db][0], hi[db][1]};
        st.o[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vw), pf, st.o[db][0], 0, 0, 0);
      }
    }
  };
  auto exp_offset = [&](float (&off)[1]) __attribute__((always_inline)) {
    off[0] = binit[0] - ((st.m_run[0] == -INFINITY) ? 0.f : st.m_run[0]);
  };

  f32x16 s0[1], s1[1];
  uint32_t p0[1][8], p1[1][8];
  float sum0[1], sum1[1], mt[1], alpha[1], off[1];
  {
    const float nb = kFastable ? -st.base[0] : 0.f;
    s0[0] = f32x16{nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb, nb};
    s1[0] = s0[0];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int ko = koff0 ^ (32 * t);  // piece 2t + lh under the swizzle: the swizzle is an exclusive or
      const bf16x8 k0 = *(const bf16x8 *)(kt + ko);
      const bf16x8 k1 = *(const bf16x8 *)(kt + 32 * G::kRow + ko);
      s0[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, st.qf[0][t], s0[0], 0, 0, 0);
      s1[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, st.qf[0][t], s1[0], 0, 0, 0);
    }
  }
  if constexpr (KEEP) {
    block_probs<1, true>(s0, 1.f, off, p0, sum0);
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(st.m_run[0] == -INFINITY) != 0, 0)) {  // (all lanes or none)
      float m = fmaxf(s0[0][0], s1[0][0]);  // (the base is still 0: these are the scores themselves)
#pragma unroll
      for (int j = 1; j < 16; ++j) m = fmaxf(m, fmaxf(s0[0][j], s1[0][j]));
      m = xhalf_max(m);
      st.m_run[0] = m, st.base[0] = m;
      off[0] = -m;
      block_probs<1, false>(s0, 1.f, off, p0, sum0);
#pragma unroll
      for (int j = 0; j < 16; ++j) s1[0][j] -= m;
    }
    if (!(sum0[0] <= kTrigger)) *(volatile int32_t *)give_up = 1;
    st.l_run[0] += sum0[0];
    pv(0, p0);
    __builtin_amdgcn_sched_barrier(0);
    block_probs<1, true>(s1, 1.f, off, p1, sum1);
    if (!(sum1[0] <= kTrigger)) *(volatile int32_t *)give_up = 1;
    st.l_run[0] += sum1[0];
    pv(1, p1);
    return;
  }
  mask_block<1, MASK>(s0, st, 0, lh, first, limit);
  if constexpr (kFastable) block_probs<1, true>(s0, 1.f, off, p0, sum0);
  block_max<1>(s0, 1.f, binit, mt);
  const bool raise0 = raise_max<1>(mt, st, alpha);
  if (!kFastable || raise0) {
    if (raise0) rescale<1>(st, alpha);
    exp_offset(off);
    block_probs<1, false>(s0, 1.f, off, p0, sum0);
  }
  st.l_run[0] += sum0[0];
  pv(0, p0);
  __builtin_amdgcn_sched_barrier(0);
  mask_block<1, MASK>(s1, st, 1, lh, first, limit);
  if constexpr (kFastable) block_probs<1, true>(s1, 1.f, off, p1, sum1);
  block_max<1>(s1, 1.f, binit, mt);
  const bool raise1 = raise_max<1>(mt, st, alpha);  // the accumulators now hold block 0 in the old units
  if (!kFastable || raise0 || raise1) {  // after a raise in block 0, S1 is no longer relative to the maximum
    if (raise1) rescale<1>(st, alpha);
    exp_offset(off);
    block_probs<1, false>(s1, 1.f, off, p1, sum1);
  }
  if (raise0 || raise1) st.base[0] = (st.m_run[0] == -INFINITY) ? 0.f : st.m_run[0];  // base == running maximum
  st.l_run[0] += sum1[0];
  pv(1, p1);
}

// The second attempt's form of the tile (see stream_tile_lean): one key block after the other, not unrolled.
template <int MASK>
__device__ __forceinline__ void stream_tile16_lean(const uint8_t *kt, RowState<1> &st, int koff0,
                                                   const int (&voff)[2][4], int lh, int first, int limit) {
  using G = Geo<false>;
  const uint8_t *vt = kt + G::kHalf;
#pragma clang loop unroll(disable)
  for (int kb = 0; kb < 2; ++kb) {
    f32x16 s[1];
    s[0] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 8; ++t)
      s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(kt + kb * 32 * G::kRow + (koff0 ^ (32 * t))),
                                                     st.qf[0][t], s[0], 0, 0, 0);
    mask_block<1, MASK>(s, st, kb, lh, first, limit);
    const float binit[1] = {0.f};
    float mt[1], alpha[1], off[1], sum[1];
    uint32_t pb[1][8];
    block_max<1>(s, 1.f, binit, mt);
    if (raise_max<1>(mt, st, alpha)) {
      rescale<1>(st, alpha);
      st.base[0] = (st.m_run[0] == -INFINITY) ? 0.f : st.m_run[0];  // base == running maximum
    }
    off[0] = -((st.m_run[0] == -INFINITY) ? 0.f : st.m_run[0]);
    block_probs<1, false>(s, 1.f, off, pb, sum);
    st.l_run[0] += sum[0];
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
      const u32x4 pw = {pb[0][4 * t2], pb[0][4 * t2 + 1], pb[0][4 * t2 + 2], pb[0][4 * t2 + 3]};
      const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
      const uint8_t *at = vt + (kb * 32 + t2 * 16) * G::kRow;
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const u32x2 lo = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((LA_LDS i16x4 *)(at + voff[0][db])));
        const u32x2 hi = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((LA_LDS i16x4 *)(at + voff[1][db])));
        const u32x4 vw = {lo[0], lo[1], hi[0], hi[1]};
        st.o[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vw), pf, st.o[db][0], 0, 0, 0);
      }
    }
  }
}

template <int NRB>
struct Stream16Shape {
  using G = Geo<false>;
  static constexpr int KSL = kWaves / NRB;
  static constexpr int kSlots = 4;                   // 128 KiB of ring
  static constexpr int NST = kSlots / KSL;
  static constexpr int IPW = 2 * G::kLoadsPerHalf * KSL / kWaves;
  static constexpr int kBlkOff = kSlots * G::kTile;
  static constexpr int kFlagOff = kBlkOff + kMaxBlkLds * 4;  // the give-up flag (see stream_tile_fast)
  static constexpr int kLdsMax = kFlagOff + 16;
  static constexpr int kFoldBytes = kWaves * 66 * 64 * 4;
  static_assert(NST >= 2 && kLdsMax <= 160 * 1024 && kFoldBytes <= kFlagOff, "LDS of one CU");
};

// The work of one workgroup; GENERAL: the second attempt, every tile in the general form (see stream_chunk).
template <int NRB, bool GENERAL>
__device__ __forceinline__ bool stream16_chunk(const AttnParams &p, uint8_t *lds, int thread_id, int block_id) {
  using S = Stream16Shape<NRB>;
  using G = Geo<false>;
  constexpr int KSL = S::KSL, NST = S::NST, IPW = S::IPW;
  constexpr int NT = 64 * kWaves;
  constexpr int kTileM = 32 * NRB;
  constexpr int kStepBytes = KSL * G::kTile;
  const int tid = thread_id;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ln = lane & 31, lh = lane >> 5;
  const int rb = wave % NRB, ks = wave / NRB;

  int id = block_id;
  const int kvh = __builtin_amdgcn_readfirstlane(id % p.Hkv);
  id = __builtin_amdgcn_readfirstlane(id / p.Hkv);
  const int row_tile = __builtin_amdgcn_readfirstlane(id % p.n_row_tiles);
  const ChunkSel sel = attn_select_chunk(p, __builtin_amdgcn_readfirstlane(id / p.n_row_tiles));
  const int b = sel.b, n_chunks = sel.n_chunks, c = sel.c, k_begin = sel.k_begin, k_end = sel.k_end;
  const int n_pre_tiles = (k_end - k_begin + kTileN - 1) / kTileN;
  const int n_pre_steps = (n_pre_tiles + KSL - 1) / KSL;
  const int n_full_steps = (k_end - k_begin) / (KSL * kTileN);

  const int r0 = row_tile * kTileM;
  const int r1 = min(p.R, r0 + kTileM);
  const int gl = p.gamma * p.L;
  const int t_lo = __builtin_amdgcn_readfirstlane(r0 / p.G), t_hi = __builtin_amdgcn_readfirstlane((r1 - 1) / p.G);
  const int tk0 = __builtin_amdgcn_readfirstlane((t_lo / p.L) * p.L);
  const int n_priv = (c == n_chunks - 1) ? (t_hi - tk0 + 1 + kTileN - 1) / kTileN : 0;
  const int n_steps = n_pre_steps + (n_priv + KSL - 1) / KSL;

  // ---- Q -> registers (before the stream starts, so that the only vector memory operations in flight later are
  //      the direct loads the kernel counts itself), times the score scale in log2 units, rounded to bf16 again
  RowState<1> st;
  const int row = r0 + rb * 32 + ln;
  {
    const int rr = min(row, p.R - 1);
    st.row_tok[0] = rr / p.G;
    st.row_bstart[0] = (st.row_tok[0] / p.L) * p.L;
    const uint8_t *qrow =
        (const uint8_t *)p.q + (((size_t)b * gl + st.row_tok[0]) * p.Hq + kvh * p.G + (rr % p.G)) * (size_t)(kD * 2);
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      u32x4 v = *(const u32x4 *)(qrow + (16 * t + 8 * lh) * 2);
      if (row >= p.R) v = u32x4{0, 0, 0, 0};
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t word = v[w];
        const uint32_t wl = word << 16, wh = word & 0xffff0000u;
        v[w] = pack_bf16(__builtin_bit_cast(float, wl) * p.scale_log2, __builtin_bit_cast(float, wh) * p.scale_log2);
      }
      st.qf[0][t] = __builtin_bit_cast(bf16x8, v);
    }
    st.m_run[0] = -INFINITY, st.l_run[0] = 0.f, st.base[0] = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int j = 0; j < 16; ++j) st.o[db][0][j] = 0.f;
  }

  // ---- physical block ids of this chunk -> LDS (paged caches only) ------------------------------
  int32_t *give_up = (int32_t *)(lds + S::kFlagOff);
  if (tid == 0) *give_up = GENERAL ? 0 : p.force_again;  // (published by the barrier below)
  int32_t *blk_lds = (int32_t *)(lds + S::kBlkOff);
  const int first_lb = k_begin >> p.block_shift;
  const int32_t *table = p.block_tables ? p.block_tables + (size_t)b * p.max_blocks : nullptr;
  if (table && k_end > k_begin) {
    const int n_blk = ((k_end - 1) >> p.block_shift) - first_lb + 1;  // <= kMaxBlkLds (host guarantees)
    for (int i = tid; i < n_blk; i += NT) blk_lds[i] = table[first_lb + i];
  }
  __syncthreads();  // (also: every wavefront holds its Q, nothing else is in flight)
  const uint32_t lds0 = (uint32_t)(size_t)(LA_LDS uint8_t *)lds;

  const size_t br_off = ((size_t)b * gl * p.Hkv + kvh) * G::kRow;
  StreamLoader<KSL, NST, IPW, false> ld;
  ld.ring = lds0, ld.wave = wave;
  ld.blk = table ? blk_lds : nullptr, ld.table = table;
  ld.first_lb = first_lb, ld.ident = b * p.max_blocks, ld.shift = p.block_shift, ld.bs_mask = p.block_size - 1;
  ld.blk_stride = (uint32_t)((p.Hkv << p.block_shift) * G::kRow), ld.br_stride = (uint32_t)(p.Hkv * G::kRow);
  ld.k_pre = (const uint8_t *)p.k_cache + ((size_t)kvh << p.block_shift) * G::kRow;
  ld.v_pre = (const uint8_t *)p.v_cache + ((size_t)kvh << p.block_shift) * G::kRow;
  ld.k_br = (const uint8_t *)p.k_branch + br_off;
  ld.v_br = (const uint8_t *)p.v_branch + br_off;
  ld.init_lane(lane);
  auto issue = [&](int step) __attribute__((always_inline)) {
    const int slot = step % NST;
    if (step < n_full_steps)
      ld.template issue<true, false>(slot, k_begin + step * (KSL * kTileN), 0);
    else if (step < n_pre_steps)
      ld.template issue<true, true>(slot, k_begin + step * (KSL * kTileN), k_end - 1);
    else
      ld.template issue<false, true>(slot, tk0 + (step - n_pre_steps) * (KSL * kTileN), t_hi);
  };
  for (int s = 0; s < NST - 1; ++s)
    if (s < n_steps) issue(s);

  int koff0, voff[2][4];
  {
    koff0 = ln * G::kRow + ((lh ^ swz_16(ln)) * 16);  // keys ln and 32 + ln share the swizzle
    // transposing read: the 16 lanes of a group address four keys x four 8-byte pieces (two neighbouring 16-byte
    // slots); lane i of the group then holds column i of those four keys
    const int grp = lane >> 4, a = lane & 15, j = a >> 2, cc = a & 3;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int keyl = 8 * half + 4 * (grp >> 1) + j;
      const int sv = swz_16(keyl);
#pragma unroll
      for (int db = 0; db < 4; ++db)
        voff[half][db] = keyl * G::kRow + (((4 * db + 2 * (grp & 1) + (cc >> 1)) ^ sv) * 16) + 8 * (cc & 1);
    }
  }

  const bool active = r0 + rb * 32 < p.R;
  int step = 0;
  if constexpr (!GENERAL) {  // the steps all of whose tiles are full prefix tiles, in a loop of their own
    for (; step < n_full_steps; ++step) {
      wait_later<IPW, NST - 2>(min(n_steps - 1, step + NST - 2) - step);
      __builtin_amdgcn_s_barrier();
      if (step + NST - 1 < n_steps) issue(step + NST - 1);
      if (active)
        stream_tile16<MASK_NONE, true>(lds + (step % NST) * kStepBytes + ks * G::kTile, st, koff0, voff, lh, 0, 0, give_up);
    }
  }
  for (; step < n_steps; ++step) {
    wait_later<IPW, NST - 2>(min(n_steps - 1, step + NST - 2) - step);
    __builtin_amdgcn_s_barrier();
    if (step + NST - 1 < n_steps) issue(step + NST - 1);
    if (!active) continue;
    const uint8_t *kt = lds + (step % NST) * kStepBytes + ks * G::kTile;
    if (step < n_pre_steps) {
      const int first = k_begin + (step * KSL + ks) * kTileN;
      if constexpr (GENERAL) {
        if (first < k_end) stream_tile16_lean<MASK_TAIL>(kt, st, koff0, voff, lh, first, k_end);
      } else {
        if (first + kTileN <= k_end)
          stream_tile16<MASK_NONE, true>(kt, st, koff0, voff, lh, 0, 0, give_up);
        else if (first < k_end)
          stream_tile16<MASK_TAIL>(kt, st, koff0, voff, lh, first, k_end);
      }
    } else {
      const int first = tk0 + ((step - n_pre_steps) * KSL + ks) * kTileN;
      if (first <= t_hi) {
        if constexpr (GENERAL)
          stream_tile16_lean<MASK_BRANCH>(kt, st, koff0, voff, lh, first, 0);
        else
          stream_tile16<MASK_BRANCH>(kt, st, koff0, voff, lh, first, 0);
      }
    }
  }
  wait_vmcnt<0>();  // no direct load may still be on its way to LDS when the workgroup gives its LDS back
  if constexpr (!GENERAL) {
    __syncthreads();  // every wavefront's flag store has landed before anyone reads the flag
    if (__builtin_expect(*(volatile int32_t *)give_up != 0, 0)) return false;
  }

  // ---- the partial: one key slice per row block writes its registers, two are folded through LDS first ---------
  const size_t slot = (size_t)b * p.s_max + c;
  const size_t out_row = slot * p.n_rows + (size_t)st.row_tok[0] * p.Hq + kvh * p.G + (row % p.G);
  float *po = p.part_o + out_row * kD;
  if constexpr (KSL > 1) {
    __builtin_amdgcn_s_barrier();
    float *fold = (float *)lds;
    if (ks > 0) {
      float *dst = fold + (size_t)((ks - 1) * NRB + rb) * 66 * 64 + lane;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int j = 0; j < 16; ++j) dst[(db * 16 + j) * 64] = st.o[db][0][j];
      dst[64 * 64] = st.m_run[0];
      dst[65 * 64] = st.l_run[0];
    }
    __syncthreads();
    if (ks > 0) return true;
#pragma unroll 1
    for (int s = 1; s < KSL; ++s) {
      const float *src = fold + (size_t)((s - 1) * NRB + rb) * 66 * 64 + lane;
      const float m2 = src[64 * 64], l2 = src[65 * 64];
      const float m_new = fmaxf(st.m_run[0], m2);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float a1 = __builtin_amdgcn_exp2f(st.m_run[0] - m_use);
      const float a2 = __builtin_amdgcn_exp2f(m2 - m_use);
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int j = 0; j < 16; ++j) st.o[db][0][j] = st.o[db][0][j] * a1 + src[(db * 16 + j) * 64] * a2;
      st.l_run[0] = st.l_run[0] * a1 + l2 * a2;
      st.m_run[0] = m_new;
    }
  }
  const float l_tot = xhalf_sum(st.l_run[0]);
  if (row < p.R) {
    // accumulator register j of d block db is head-dim column 32*db + 8*(j/4) + 4*lh + j%4
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 v = {st.o[db][0][4 * q], st.o[db][0][4 * q + 1], st.o[db][0][4 * q + 2], st.o[db][0][4 * q + 3]};
        *(f32x4 *)(po + 32 * db + 8 * q + 4 * lh) = v;
      }
    if (lh == 0) {
      const f32x2 ml = {st.m_run[0], l_tot};
      *(f32x2 *)(p.part_ml + out_row * 2) = ml;
    }
  }
  return true;
}

template <int NRB>
__global__ __launch_bounds__(64 * kWaves) void attn_stream16_kernel(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  if (__builtin_expect(!stream16_chunk<NRB, false>(p, lds, threadIdx.x, blockIdx.x), 0)) {
    int thread_id = threadIdx.x, block_id = blockIdx.x;  // (opaque to the compiler: see attn_stream_kernel)
    asm volatile("" : "+v"(thread_id), "+s"(block_id));
    stream16_chunk<NRB, true>(p, lds, thread_id, block_id);
  }
}

template <int NRB>
hipError_t launch_stream16_variant(const AttnParams &p, hipStream_t stream) {
  using S = Stream16Shape<NRB>;
  const int grid = p.Hkv * p.n_row_tiles * p.total_units;
  auto kern = attn_stream16_kernel<NRB>;
  const int blk_entries =
      p.block_tables ? (attn_max_chunk_tokens(p.chunk_len, p.last_short) >> p.block_shift) + 2 : 0;
  if (blk_entries > kMaxBlkLds) return hipErrorInvalidValue;
  const int lds_bytes = S::kLdsMax;  // (the flag lies behind the largest block table)
  static std::once_flag once;
  static hipError_t configured = hipSuccess;
  std::call_once(once, [&] {
    configured = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, S::kLdsMax);
  });
  if (configured != hipSuccess) return configured;
  AttnParams q = p;
  q.force_again = selftest_force_second_attempt ? selftest_force_second_attempt() : 0;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * kWaves), lds_bytes, stream, q);
  return hipGetLastError();
}

template <int NRB>
hipError_t launch_stream_variant(const AttnParams &p, hipStream_t stream) {
  using S = StreamShape<NRB>;
  const int grid = p.Hkv * p.n_row_tiles * p.total_units;
  auto kern = attn_stream_kernel<NRB>;
  const int blk_entries =
      p.block_tables ? (attn_max_chunk_tokens(p.chunk_len, p.last_short) >> p.block_shift) + 2 : 0;
  if (blk_entries > kMaxBlkLds) return hipErrorInvalidValue;
  const int lds_bytes = S::kBlkOff + blk_entries * 4 > S::kFoldBytes ? S::kBlkOff + blk_entries * 4 : S::kFoldBytes;
  static std::once_flag once;
  static hipError_t configured = hipSuccess;
  std::call_once(once, [&] {
    configured = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, S::kLdsMax);
  });
  if (configured != hipSuccess) return configured;
  AttnParams q = p;
  q.force_again = selftest_force_second_attempt ? selftest_force_second_attempt() : 0;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * kWaves), lds_bytes, stream, q);
  return hipGetLastError();
}

// row blocks per workgroup of the shapes: three for an fp8 cache, then two for a bf16 cache
constexpr int kStreamNrb[] = {2, 4, 8, 8, 4};
constexpr int kNumStreamShapes = 5;

}  // namespace

int attn_stream_num_shapes() { return kNumStreamShapes; }
int attn_stream_tile_m(int shape) { return 32 * kStreamNrb[shape]; }
int attn_stream_step_keys(int shape) { return kTileN * kWaves / kStreamNrb[shape]; }
int attn_stream_max_chunk_blocks() { return kMaxBlkLds; }
bool attn_stream_shape_is_fp8(int shape) { return shape < 3; }

hipError_t launch_attn_stream(const AttnParams &p, int shape, hipStream_t stream) {
  ProfileScope scope(SLOT_ATTN_MFMA, stream);
  switch (shape) {
    case 0: return launch_stream_variant<2>(p, stream);
    case 1: return launch_stream_variant<4>(p, stream);
    case 2: return launch_stream_variant<8>(p, stream);
    case 3: return launch_stream16_variant<8>(p, stream);
    case 4: return launch_stream16_variant<4>(p, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace la
