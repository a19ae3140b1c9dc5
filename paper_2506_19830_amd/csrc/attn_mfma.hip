// Shared-prefix verify attention, bf16 MFMA path (gfx950).
//
// The verification pass expands all drafted branches against one shared prefix
// (Algorithm 1, "in parallel do"; prefixes x'_j).  Here the R = gamma*L*G query
// rows that share a KV head are tiled into row tiles; a workgroup owns
// (row tile, kv head, prefix chunk), streams the chunk's K/V tiles through LDS
// once and reuses every tile for all its rows.  The workgroup that owns the last
// chunk of a request also reduces the branch-private keys under the mask
// "same branch and key position <= query position".
//
// Per 64-key tile and wavefront (RB blocks of 32 rows each):
//   S^T = K Q^T      v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q (registers)
//   online softmax   each lane owns one query row (column of S^T): the row max is an
//                    in-lane reduction plus one exchange with lane^32
//   O^T += V^T P^T   A = V^T from LDS (stored transposed, keys permuted inside groups
//                    of 16 so that the accumulator registers of S^T are already the
//                    B operand; row 32*db + m of the LDS tile holds head-dim column
//                    4*m + db, which makes the transposing LDS writes bank-conflict
//                    free and the four db accumulators of a lane adjacent columns),
//                    B = P^T (registers, bf16)
// Everything is kept in log2 units: p = 2^(s*c - m).
#include "la_internal.hpp"

namespace la {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kD = 128;                      // head dim
constexpr int kTileN = 64;                   // keys per tile
constexpr int kKRow = kD * 2 + 16;           // bytes per key row of the K tile in LDS (padded)
constexpr int kVRow = kTileN * 2 + 16;       // bytes per d row of the V^T tile in LDS (padded)
constexpr int kKTileBytes = kTileN * kKRow;  // 17408
constexpr int kVTileBytes = kD * kVRow;      // 18432
constexpr int kStageBytes = kKTileBytes + kVTileBytes;
constexpr int kMaxChunkBlocks = 4096;        // block ids of one chunk kept in LDS
constexpr int kStages = 3;                   // LDS ring: tile i is computed on while i+1 is resident and i+2 is written
constexpr int kLdsTotal = kStages * kStageBytes + kMaxChunkBlocks * 4;  // stages + block ids: 123904

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}

// two fp8-e4m3 of a 32-bit word (low or high half) -> a bf16 pair (exact), scale factor 1
template <bool HI>
__device__ __forceinline__ uint32_t fp8x2_to_bf16x2(uint32_t w) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, HI));
}

// position of key quad kq (keys 4kq..4kq+3 of the tile) inside a V^T row: inside every group of 16 keys
// key 8a+4h+c sits at 8h+4a+c, which is the order the S^T accumulator registers come in
__device__ __forceinline__ int vt_pos(int kq) { return 16 * (kq >> 2) + 8 * (kq & 1) + 4 * ((kq >> 1) & 1); }

// LDS row of head-dim column d in the V^T tile: block d%4, row d/4 inside the block
__device__ __forceinline__ int vt_row(int d) { return (d & 3) * 32 + (d >> 2); }
// bf16 V loads: lane -> column pair so that lanes 0..31 hold the even pairs and lanes 32..63 the odd ones; the
// transposed LDS writes of a half wavefront then land in consecutive rows
__device__ __forceinline__ int v_pair_of_lane(int lane) { return 2 * (lane & 31) + (lane >> 5); }

// max / sum of a value with its partner in the other half of the wavefront (lane ^ 32)
__device__ __forceinline__ float xhalf_max(float v) {
  const uint32_t u = __builtin_bit_cast(uint32_t, v);
  const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const uint32_t a = sw[0], b = sw[1];
  return fmaxf(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b));
}
__device__ __forceinline__ float xhalf_sum(float v) {
  const uint32_t u = __builtin_bit_cast(uint32_t, v);
  const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const uint32_t a = sw[0], b = sw[1];
  return __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b);
}

// Where the keys of one tile come from.
struct TileSrc {
  const uint8_t *k_base, *v_base;  // prefix: cache base of this kv head; branch: row of token 0 of this request/head
  const int32_t *blk;              // prefix: physical block ids of this chunk (LDS), indexed from first_lb
  int first_lb;                    // prefix: logical block of blk[0]
  int first;                       // first key of the tile (prefix: token index; branch: token t = g*L+j)
  int limit;                       // keys >= limit are zero filled
};

// Staging registers of one K tile and one V tile per thread: 16-byte pieces of K rows, 4-byte pieces of V rows.
template <bool FP8, int NT>
struct TileRegs {
  static constexpr int kNK = (FP8 ? 512 : 1024) / NT;  // K pieces per thread
  static constexpr int kNV = (FP8 ? 512 : 1024) / NT;  // V key quads per thread
  u32x4 k[kNK];
  uint32_t v[4 * kNV];
};

// Address of key row `tok`.  Cache blocks are [block][Hkv][block_size][D]: inside a block consecutive tokens of
// one head are contiguous.
template <bool FP8, bool PREFIX>
__device__ __forceinline__ const uint8_t *key_row(const AttnParams &p, const TileSrc &s, const uint8_t *base,
                                                  int tok) {
  constexpr int row_bytes = kD * (FP8 ? 1 : 2);
  if constexpr (PREFIX) {
    const int blk = s.blk[(tok >> p.block_shift) - s.first_lb];
    return base + (((size_t)blk * p.Hkv) << p.block_shift) * row_bytes +
           (size_t)(tok & (p.block_size - 1)) * row_bytes;
  }
  return base + (size_t)tok * p.Hkv * row_bytes;
}

// Global -> registers.  FULL: every key of the tile is below s.limit.  Otherwise addresses are clamped to the
// last valid key and the values zeroed, so the loads stay unconditional and in bounds.
template <bool FP8, bool PREFIX, bool FULL, int NT>
__device__ __forceinline__ void tile_load(const AttnParams &p, const TileSrc &s, int tid, TileRegs<FP8, NT> &r) {
  constexpr int row_bytes = kD * (FP8 ? 1 : 2);
  constexpr int k_piece_shift = FP8 ? 3 : 4;  // 16-byte pieces per key row: 8 (fp8) or 16 (bf16)
#pragma unroll
  for (int e = 0; e < TileRegs<FP8, NT>::kNK; ++e) {
    const int idx = tid + NT * e;
    const int tok = s.first + (idx >> k_piece_shift);
    const int tc = FULL ? tok : min(tok, s.limit - 1);
    u32x4 val = *(const u32x4 *)(key_row<FP8, PREFIX>(p, s, s.k_base, tc) + (idx & ((1 << k_piece_shift) - 1)) * 16);
    if (!FULL && tok >= s.limit) val = u32x4{0, 0, 0, 0};
    r.k[e] = val;
  }
  constexpr int v_quad_shift = FP8 ? 5 : 6;  // 4-byte pieces per key row: 32 (fp8) or 64 (bf16)
#pragma unroll
  for (int e = 0; e < TileRegs<FP8, NT>::kNV; ++e) {
    const int idx = tid + NT * e;
    const int kq = idx >> v_quad_shift;
    const int piece = FP8 ? (idx & 31) : v_pair_of_lane(idx & 63);
    const int tok0 = s.first + 4 * kq;  // the four keys of a quad share a cache block (block_size % 16 == 0)
    if constexpr (FULL && PREFIX) {
      const uint8_t *row = key_row<FP8, PREFIX>(p, s, s.v_base, tok0) + piece * 4;
#pragma unroll
      for (int c = 0; c < 4; ++c) r.v[4 * e + c] = *(const uint32_t *)(row + c * row_bytes);
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int tok = tok0 + c;
        const int tc = min(tok, s.limit - 1);
        const uint32_t val = *(const uint32_t *)(key_row<FP8, PREFIX>(p, s, s.v_base, tc) + piece * 4);
        r.v[4 * e + c] = tok < s.limit ? val : 0u;
      }
    }
  }
}

// Registers -> LDS stage: K rows as they are, V transposed ([d][key], keys permuted by vt_pos); fp8 is widened to
// bf16 on the way (exact: every e4m3 value is a bf16 value).
template <bool FP8, int NT>
__device__ __forceinline__ void tile_store(uint8_t *stage, int tid, const TileRegs<FP8, NT> &r) {
  uint8_t *kt = stage;
  uint8_t *vt = stage + kKTileBytes;
  if constexpr (!FP8) {
#pragma unroll
    for (int e = 0; e < TileRegs<FP8, NT>::kNK; ++e) {
      const int idx = tid + NT * e;
      *(u32x4 *)(kt + (idx >> 4) * kKRow + (idx & 15) * 16) = r.k[e];
    }
#pragma unroll
    for (int e = 0; e < TileRegs<FP8, NT>::kNV; ++e) {
      const int idx = tid + NT * e;
      const int kq = idx >> 6;
      const int dp = v_pair_of_lane(idx & 63);  // this thread holds columns 2dp, 2dp+1 of the quad's 4 keys
      const uint32_t a = r.v[4 * e + 0], b = r.v[4 * e + 1], c = r.v[4 * e + 2], d = r.v[4 * e + 3];
      // low halves hold column 2dp of keys (a,b,c,d), high halves column 2dp+1
      u32x2 lo = {__builtin_amdgcn_perm(b, a, 0x05040100u), __builtin_amdgcn_perm(d, c, 0x05040100u)};
      u32x2 hi = {__builtin_amdgcn_perm(b, a, 0x07060302u), __builtin_amdgcn_perm(d, c, 0x07060302u)};
      *(u32x2 *)(vt + vt_row(2 * dp) * kVRow + vt_pos(kq) * 2) = lo;
      *(u32x2 *)(vt + vt_row(2 * dp + 1) * kVRow + vt_pos(kq) * 2) = hi;
    }
  } else {
#pragma unroll
    for (int e = 0; e < TileRegs<FP8, NT>::kNK; ++e) {
      const int idx = tid + NT * e;
      uint32_t out[8];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t word = r.k[e][w];
        out[2 * w] = fp8x2_to_bf16x2<false>(word);
        out[2 * w + 1] = fp8x2_to_bf16x2<true>(word);
      }
      uint8_t *dst = kt + (idx >> 3) * kKRow + (idx & 7) * 32;
      *(u32x4 *)(dst) = u32x4{out[0], out[1], out[2], out[3]};
      *(u32x4 *)(dst + 16) = u32x4{out[4], out[5], out[6], out[7]};
    }
#pragma unroll
    for (int e = 0; e < TileRegs<FP8, NT>::kNV; ++e) {
      const int idx = tid + NT * e;
      const int kq = idx >> 5;
      const int d0 = 4 * (idx & 31);
      uint32_t lo[4], hi[4];  // of key c: bf16 pairs (d0, d0+1) and (d0+2, d0+3)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        lo[c] = fp8x2_to_bf16x2<false>(r.v[4 * e + c]);
        hi[c] = fp8x2_to_bf16x2<true>(r.v[4 * e + c]);
      }
      // columns d0..d0+3 live in rows (d0/4) + 32*{0,1,2,3}: consecutive lanes write consecutive rows
      uint8_t *dst = vt + (d0 >> 2) * kVRow + vt_pos(kq) * 2;
      // column d0: low halves of lo[0..3]; column d0+1: high halves; columns d0+2, d0+3 likewise from hi[]
      *(u32x2 *)(dst) = u32x2{__builtin_amdgcn_perm(lo[1], lo[0], 0x05040100u),
                              __builtin_amdgcn_perm(lo[3], lo[2], 0x05040100u)};
      *(u32x2 *)(dst + 32 * kVRow) = u32x2{__builtin_amdgcn_perm(lo[1], lo[0], 0x07060302u),
                                           __builtin_amdgcn_perm(lo[3], lo[2], 0x07060302u)};
      *(u32x2 *)(dst + 64 * kVRow) = u32x2{__builtin_amdgcn_perm(hi[1], hi[0], 0x05040100u),
                                           __builtin_amdgcn_perm(hi[3], hi[2], 0x05040100u)};
      *(u32x2 *)(dst + 96 * kVRow) = u32x2{__builtin_amdgcn_perm(hi[1], hi[0], 0x07060302u),
                                           __builtin_amdgcn_perm(hi[3], hi[2], 0x07060302u)};
    }
  }
}

// A running maximum is only raised when the tile maximum exceeds it by more than this many log2 units; until
// then probabilities are allowed to reach 2^kRaise, which fp32 sums and bf16 operands hold without loss.  Raising
// rarely keeps the accumulator rescale (64 multiplies per lane and row block) off the common path.
constexpr float kRaise = 6.0f;

// Per-wavefront state of RB blocks of 32 query rows.
template <int RB>
struct RowState {
  bf16x8 qf[RB][8];  // Q^T operand: row ln of block rb, d = 16t + 8*lh .. +8
  f32x16 o[4][RB];   // O^T accumulators: d block db, row block rb
  float m_run[RB], l_run[RB];
  int row_tok[RB], row_bstart[RB];
};

enum MaskMode { MASK_NONE = 0, MASK_TAIL = 1, MASK_BRANCH = 2 };

// sched_group_barrier masks
constexpr int kSgMfma = 0x008, kSgValu = 0x002, kSgDsRead = 0x100;

// Mask the scores of one 32-key block: register j holds key  kb*32 + (j/4)*8 + lh*4 + j%4  of the tile.
template <int RB, int MASK>
__device__ __forceinline__ void mask_block(f32x16 (&s)[RB], const RowState<RB> &st, int kb, int lh, int first,
                                           int limit) {
  if constexpr (MASK == MASK_TAIL) {
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int key = first + kb * 32 + (j >> 2) * 8 + lh * 4 + (j & 3);
      if (key >= limit) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) s[rb][j] = -INFINITY;
      }
    }
  } else if constexpr (MASK == MASK_BRANCH) {
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int tk = first + kb * 32 + (j >> 2) * 8 + lh * 4 + (j & 3);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        if (tk > st.row_tok[rb] || tk < st.row_bstart[rb]) s[rb][j] = -INFINITY;
    }
  }
}

// Fold the block maximum of every row into its running maximum (log2 units).  A lane raises its maximum only when
// the block exceeds it by more than kRaise; alpha is the factor its old accumulators must then be multiplied by
// (1 for lanes that keep their maximum).  Returns whether any lane of the wavefront raised (wavefront-uniform).
template <int RB>
__device__ __forceinline__ bool update_max(const f32x16 (&s)[RB], RowState<RB> &st, float cseg, float (&alpha)[RB]) {
  bool raise = false;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float m0 = fmaxf(s[rb][0], s[rb][1]);
#pragma unroll
    for (int j = 2; j < 16; j += 2) m0 = fmaxf(m0, fmaxf(s[rb][j], s[rb][j + 1]));
    const float mt = xhalf_max(m0) * cseg;
    const bool up = mt > st.m_run[rb] + kRaise;   // false for mt = -inf; true for the first finite block (m_run = -inf)
    const float m_new = up ? mt : st.m_run[rb];
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    alpha[rb] = up ? __builtin_amdgcn_exp2f(st.m_run[rb] - m_use) : 1.0f;   // 0 when m_run was -inf
    st.m_run[rb] = m_new;
    raise |= up;
  }
  return __builtin_amdgcn_ballot_w64(raise) != 0;
}

template <int RB>
__device__ __forceinline__ void rescale(RowState<RB> &st, const float (&alpha)[RB]) {
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    st.l_run[rb] *= alpha[rb];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int j = 0; j < 16; ++j) st.o[db][rb][j] *= alpha[rb];
  }
}

// p = 2^(s*cseg - m + voff) for one 32-key block, rounded to bf16 pairs; also the fp32 row sums.
template <int RB>
__device__ __forceinline__ void block_probs(const f32x16 (&s)[RB], const RowState<RB> &st, float cseg, float voff,
                                            uint32_t (&pb)[RB][8], float (&sum)[RB]) {
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const float m_use = (st.m_run[rb] == -INFINITY) ? 0.f : st.m_run[rb];
    const float off = voff - m_use;
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < 16; j += 2) {
#ifdef LA_EXP_NOEXP
      const float p0 = __builtin_fmaf(s[rb][j], cseg, off);
      const float p1 = __builtin_fmaf(s[rb][j + 1], cseg, off);
#else
      const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[rb][j], cseg, off));
      const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[rb][j + 1], cseg, off));
#endif
      pb[rb][j >> 1] = pack_bf16(p0, p1);
      // (a v_dot2c_f32_bf16 on the packed pair would sum the rounded values in one instruction, but on gfx950 it
      // stalls against the MFMAs in flight: measured slower than the two adds)
      acc += p0 + p1;
    }
    sum[rb] = acc;
  }
}

// One 64-key tile from an LDS stage, as two 32-key blocks whose MFMA and VALU work is interleaved:
//     S0 = K0 Q^T                    |
//     S1 = K1 Q^T                    |  P0 = 2^(S0 - m)          (VALU next to the MFMAs of the other block)
//     O += V0^T P0                   |  P1 = 2^(S1 - m)
//     O += V1^T P1                   |  tail()  (the caller's LDS stores of the next tile)
//   first / limit   MASK_TAIL: keys with first + key >= limit are masked
//                   MASK_BRANCH: key token first + key is visible to a row iff row_bstart <= token <= row_tok
//   cseg            score scale of this key segment (log2 units); voff/lmul move a differently scaled V segment into
//                   the accumulator's units (p' = p * 2^voff, l += sum(p') * lmul)
//   k0              the K fragments of key block 0.  K0_READY: the caller already holds them (fetched while the
//                   previous tile was finishing); otherwise they are read here.  With next_kt != nullptr the block-0
//                   fragments of the tile staged at next_kt are fetched behind the last MFMAs and left in k0.
template <int RB, int MASK, bool K0_READY, bool PREFETCH, typename Tail>
__device__ __forceinline__ void compute_tile(const uint8_t *kt, const uint8_t *next_kt, bf16x8 (&k0)[8],
                                             RowState<RB> &st, int ln, int lh, int first, int limit, float cseg,
                                             float voff, float lmul, Tail &&tail) {
  const uint8_t *krow = kt + ln * kKRow + lh * 16;
  const uint8_t *vrow = kt + kKTileBytes + ln * kVRow + lh * 16;
  auto load_k = [&](int t, int kb) {
    return __builtin_bit_cast(bf16x8, *(const u32x4 *)(krow + kb * 32 * kKRow + t * 32));
  };
  auto load_v = [&](int db, int kb, int t2) {
    return __builtin_bit_cast(bf16x8, *(const u32x4 *)(vrow + db * 32 * kVRow + (kb * 32 + t2 * 16) * 2));
  };
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // ---- S0 = K0 Q^T; the K1 fragments are fetched behind the MFMAs ---------------------------
  f32x16 s0[RB], s1[RB];
  bf16x8 k1[8];
  if constexpr (!K0_READY) {
#pragma unroll
    for (int t = 0; t < 8; ++t) k0[t] = load_k(t, 0);
  }
#pragma unroll
  for (int t = 0; t < 8; ++t) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      s0[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0[t], st.qf[rb][t], t == 0 ? zero : s0[rb], 0, 0, 0);
    k1[t] = load_k(t, 1);
  }
  if constexpr (!K0_READY) __builtin_amdgcn_sched_group_barrier(kSgDsRead, 8, 0);
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    __builtin_amdgcn_sched_group_barrier(kSgMfma, RB, 0);
    __builtin_amdgcn_sched_group_barrier(kSgDsRead, 1, 0);
  }
  mask_block<RB, MASK>(s0, st, 0, lh, first, limit);
  float alpha[RB];
  if (update_max<RB>(s0, st, cseg, alpha)) rescale<RB>(st, alpha);

  // ---- one basic block: S1 = K1 Q^T next to P0 = 2^(S0 - m), then O += V0^T P0 next to P1 = 2^(S1 - m).
  //      The V fragments are fetched from LDS behind the MFMAs.
  uint32_t p0[RB][8], p1[RB][8];
  float sum0[RB], sum1[RB];
  bf16x8 v0[2][4], v1[2][4];
#pragma unroll
  for (int t = 0; t < 8; ++t)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      s1[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1[t], st.qf[rb][t], t == 0 ? zero : s1[rb], 0, 0, 0);
  block_probs<RB>(s0, st, cseg, voff, p0, sum0);
#pragma unroll
  for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
    for (int db = 0; db < 4; ++db) v0[t2][db] = load_v(db, 0, t2);
#pragma unroll
  for (int i = 0; i < 8; ++i) {  // per step: RB MFMAs, 6*RB VALU (of 48*RB), one LDS read
    __builtin_amdgcn_sched_group_barrier(kSgMfma, RB, 0);
    __builtin_amdgcn_sched_group_barrier(kSgValu, 6 * RB, 0);
    __builtin_amdgcn_sched_group_barrier(kSgDsRead, 1, 0);
  }
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) st.l_run[rb] += sum0[rb] * lmul;
  mask_block<RB, MASK>(s1, st, 1, lh, first, limit);
  const bool raise1 = update_max<RB>(s1, st, cseg, alpha);  // accumulators are rescaled after block 0 went in
#pragma unroll
  for (int t2 = 0; t2 < 2; ++t2) {
    bf16x8 pf[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      u32x4 v = {p0[rb][4 * t2], p0[rb][4 * t2 + 1], p0[rb][4 * t2 + 2], p0[rb][4 * t2 + 3]};
      pf[rb] = __builtin_bit_cast(bf16x8, v);
    }
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        st.o[db][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v0[t2][db], pf[rb], st.o[db][rb], 0, 0, 0);
  }
  block_probs<RB>(s1, st, cseg, voff, p1, sum1);
#pragma unroll
  for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
    for (int db = 0; db < 4; ++db) v1[t2][db] = load_v(db, 1, t2);
  __builtin_amdgcn_sched_group_barrier(kSgValu, 14 * RB, 0);  // the block-1 maximum
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    __builtin_amdgcn_sched_group_barrier(kSgMfma, RB, 0);
    __builtin_amdgcn_sched_group_barrier(kSgValu, 6 * RB, 0);
    __builtin_amdgcn_sched_group_barrier(kSgDsRead, 1, 0);
  }
  // keep the block-1 probabilities on this side of the branch below (otherwise they are sunk past it and no longer
  // overlap the MFMAs above)
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
    asm volatile("" ::"v"(p1[rb][0]), "v"(p1[rb][1]), "v"(p1[rb][2]), "v"(p1[rb][3]), "v"(p1[rb][4]), "v"(p1[rb][5]),
                 "v"(p1[rb][6]), "v"(p1[rb][7]), "v"(sum1[rb]));
  if (raise1) rescale<RB>(st, alpha);
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) st.l_run[rb] += sum1[rb] * lmul;

  // ---- O += V1^T P1 next to the caller's tail work ----------------------------------------------
#pragma unroll
  for (int t2 = 0; t2 < 2; ++t2) {
    bf16x8 pf[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      u32x4 v = {p1[rb][4 * t2], p1[rb][4 * t2 + 1], p1[rb][4 * t2 + 2], p1[rb][4 * t2 + 3]};
      pf[rb] = __builtin_bit_cast(bf16x8, v);
    }
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        st.o[db][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v1[t2][db], pf[rb], st.o[db][rb], 0, 0, 0);
  }
  if constexpr (PREFETCH) {
    const uint8_t *nrow = next_kt + ln * kKRow + lh * 16;
#pragma unroll
    for (int t = 0; t < 8; ++t) k0[t] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(nrow + t * 32));
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      __builtin_amdgcn_sched_group_barrier(kSgMfma, RB, 0);
      __builtin_amdgcn_sched_group_barrier(kSgDsRead, 1, 0);
    }
  }
  tail();
}

// NW wavefronts of RB 32-row blocks each: a row tile of 32*NW*RB rows.
template <bool KV_FP8, bool BR_FP8, int NW, int RB>
__global__ __launch_bounds__(64 * NW, (NW * RB <= 4) ? 2 : 1) void attn_mfma_kernel(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  constexpr int NT = 64 * NW;
  constexpr int kTileM = 32 * NW * RB;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, lh = lane >> 5;

  // ---- which (kv head, row tile, request, chunk) -------------------------------------------
  int id = blockIdx.x;
  const int kvh = id % p.Hkv;
  id /= p.Hkv;
  const int row_tile = id % p.n_row_tiles;
  int c = id / p.n_row_tiles;
  int b = 0;
  for (; b < p.B - 1; ++b) {
    const int nc = attn_num_chunks(p.prefix_lens[b], p.chunk_len);
    if (c < nc) break;
    c -= nc;
  }
  const int P = p.prefix_lens[b];
  const int n_chunks = attn_num_chunks(P, p.chunk_len);
  const int k_begin = c * p.chunk_len;
  const int k_end = min(P, k_begin + p.chunk_len);
  const int n_full = k_end > k_begin ? (k_end - k_begin) / kTileN : 0;          // unmasked prefix tiles
  const bool has_tail = k_end > k_begin && ((k_end - k_begin) % kTileN) != 0;  // one partly filled prefix tile

  const int r0 = row_tile * kTileM;
  const int r1 = min(p.R, r0 + kTileM);
  const int gl = p.gamma * p.L;
  // branch-private keys needed by this row tile: tokens t = g*L + j in [tk0, t_hi]
  const int t_lo = r0 / p.G, t_hi = (r1 - 1) / p.G;
  const int tk0 = (t_lo / p.L) * p.L;
  const int n_priv = (c == n_chunks - 1) ? (t_hi - tk0 + 1 + kTileN - 1) / kTileN : 0;

  // ---- physical block ids of this chunk -> LDS ---------------------------------------------
  int32_t *blk_lds = (int32_t *)(lds + kStages * kStageBytes);
  const int first_lb = k_begin >> p.block_shift;
  if (k_end > k_begin) {
    const int n_blk = ((k_end - 1) >> p.block_shift) - first_lb + 1;  // <= kMaxChunkBlocks (host guarantees)
    const int32_t *table = p.block_tables ? p.block_tables + (size_t)b * p.max_blocks : nullptr;
    for (int i = tid; i < n_blk; i += NT)
      blk_lds[i] = table ? table[first_lb + i] : b * p.max_blocks + first_lb + i;
  }

  constexpr int kv_row = kD * (KV_FP8 ? 1 : 2);
  constexpr int br_row = kD * (BR_FP8 ? 1 : 2);
  TileSrc pre;  // prefix tiles
  pre.k_base = (const uint8_t *)p.k_cache + ((size_t)kvh << p.block_shift) * kv_row;
  pre.v_base = (const uint8_t *)p.v_cache + ((size_t)kvh << p.block_shift) * kv_row;
  pre.blk = blk_lds;
  pre.first_lb = first_lb;
  pre.limit = k_end;
  TileSrc brs;  // branch-private tiles
  const size_t br_off = ((size_t)b * gl * p.Hkv + kvh) * br_row;
  brs.k_base = (const uint8_t *)p.k_branch + br_off;
  brs.v_base = (const uint8_t *)p.v_branch + br_off;
  brs.blk = nullptr;
  brs.first_lb = 0;
  brs.limit = t_hi + 1;

  // ---- per-lane query rows ---------------------------------------------------------------
  RowState<RB> st;
  int row[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int r = r0 + (wave * RB + rb) * 32 + ln;
    row[rb] = r;
    const int rr = min(r, p.R - 1);
    st.row_tok[rb] = rr / p.G;
    st.row_bstart[rb] = (st.row_tok[rb] / p.L) * p.L;
    const uint8_t *qrow =
        (const uint8_t *)p.q + (((size_t)b * gl + st.row_tok[rb]) * p.Hq + kvh * p.G + (rr % p.G)) * (size_t)(kD * 2);
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      u32x4 v = *(const u32x4 *)(qrow + (16 * t + 8 * lh) * 2);
      if (r >= p.R) v = u32x4{0, 0, 0, 0};
      st.qf[rb][t] = __builtin_bit_cast(bf16x8, v);
    }
    st.m_run[rb] = -INFINITY;
    st.l_run[rb] = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int j = 0; j < 16; ++j) st.o[db][rb][j] = 0.f;
  }

  // scale factors of the two key segments, in log2 units
  float c_prefix = p.scale_log2, c_branch = p.scale_log2;
  float vmul_branch = 1.0f;  // branch V is multiplied by this to live in the prefix segment's V units
  float v_out = 1.0f;
  if (KV_FP8) {
    const float ks = p.k_scale ? p.k_scale[kvh] : 1.0f;
    const float vs = p.v_scale ? p.v_scale[kvh] : 1.0f;
    c_prefix *= ks;
    v_out = vs;
    if (BR_FP8)
      c_branch *= ks;
    else
      vmul_branch = 1.0f / vs;
  }
  const float voff_branch = __builtin_log2f(vmul_branch);
  const float lmul_branch = 1.0f / vmul_branch;

  __syncthreads();  // block ids visible

  // ---- phase 1: the unmasked prefix tiles through a ring of three LDS stages ----------------------
  // iteration i: global loads of tile i+2 are in flight, tile i is computed from stage i%3 (its block-0 K fragments
  // were fetched while tile i-1 finished), the block-0 fragments of tile i+1 are fetched from stage (i+1)%3, and
  // tile i+2 is written to stage (i+2)%3, which every wavefront stopped reading at the barrier before.
  bf16x8 k0[8];
  if (n_full > 0) {
    TileRegs<KV_FP8, NT> regs;
    auto stage_of = [&](int it) { return lds + (it % kStages) * kStageBytes; };
    auto gload = [&](int it) {
      pre.first = k_begin + it * kTileN;
      tile_load<KV_FP8, true, true, NT>(p, pre, tid, regs);
    };
    gload(0);
    tile_store<KV_FP8, NT>(stage_of(0), tid, regs);
    if (n_full > 1) {
      gload(1);
      tile_store<KV_FP8, NT>(stage_of(1), tid, regs);
    }
    __syncthreads();
    {
      const uint8_t *krow = stage_of(0) + ln * kKRow + lh * 16;
#pragma unroll
      for (int t = 0; t < 8; ++t) k0[t] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(krow + t * 32));
    }
    int it = 0;
    for (; it + 2 < n_full; ++it) {  // steady state: nothing conditional
      gload(it + 2);
      compute_tile<RB, MASK_NONE, true, true>(stage_of(it), stage_of(it + 1), k0, st, ln, lh, 0, 0, c_prefix, 0.f,
                                              1.f, [&] { tile_store<KV_FP8, NT>(stage_of(it + 2), tid, regs); });
      __syncthreads();
    }
    if (it + 1 < n_full) {  // second to last tile: nothing left to load
      compute_tile<RB, MASK_NONE, true, true>(stage_of(it), stage_of(it + 1), k0, st, ln, lh, 0, 0, c_prefix, 0.f,
                                              1.f, [] {});
      ++it;
    }
    compute_tile<RB, MASK_NONE, true, false>(stage_of(it), nullptr, k0, st, ln, lh, 0, 0, c_prefix, 0.f, 1.f, [] {});
    __syncthreads();
  }
  // ---- phase 2: the partly filled prefix tile -------------------------------------------------
  if (has_tail) {
    TileRegs<KV_FP8, NT> regs;
    pre.first = k_begin + n_full * kTileN;
    tile_load<KV_FP8, true, false, NT>(p, pre, tid, regs);
    tile_store<KV_FP8, NT>(lds, tid, regs);
    __syncthreads();
    compute_tile<RB, MASK_TAIL, false, false>(lds, nullptr, k0, st, ln, lh, pre.first, k_end, c_prefix, 0.f, 1.f,
                                              [] {});
    __syncthreads();
  }
  // ---- phase 3: branch-private tiles (last chunk only) ------------------------------------------
  for (int it = 0; it < n_priv; ++it) {
    TileRegs<BR_FP8, NT> regs;
    brs.first = tk0 + it * kTileN;
    tile_load<BR_FP8, false, false, NT>(p, brs, tid, regs);
    tile_store<BR_FP8, NT>(lds, tid, regs);
    __syncthreads();
    compute_tile<RB, MASK_BRANCH, false, false>(lds, nullptr, k0, st, ln, lh, brs.first, 0, c_branch, voff_branch,
                                                lmul_branch, [] {});
    __syncthreads();
  }

  // ---- write the partial -----------------------------------------------------------------
  const size_t slot = (size_t)b * p.s_max + c;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const float l_tot = xhalf_sum(st.l_run[rb]);
    if (row[rb] < p.R) {
      const size_t out_row = slot * p.n_rows + (size_t)st.row_tok[rb] * p.Hq + kvh * p.G + (row[rb] % p.G);
      float *po = p.part_o + out_row * kD;
      // accumulator register j of d block db is MFMA row m = 8*(j/4) + 4*lh + j%4, i.e. column 4m + db
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int m = 8 * (j >> 2) + 4 * lh + (j & 3);
        f32x4 v = {st.o[0][rb][j] * v_out, st.o[1][rb][j] * v_out, st.o[2][rb][j] * v_out, st.o[3][rb][j] * v_out};
        *(f32x4 *)(po + 4 * m) = v;
      }
      if (lh == 0) {
        f32x2 ml = {st.m_run[rb], l_tot};
        *(f32x2 *)(p.part_ml + out_row * 2) = ml;
      }
    }
  }
}

template <bool KV_FP8, bool BR_FP8, int NW, int RB>
hipError_t launch_variant(const AttnParams &p, hipStream_t stream) {
  const int grid = p.Hkv * p.n_row_tiles * p.total_units;
  auto kern = attn_mfma_kernel<KV_FP8, BR_FP8, NW, RB>;
  static bool configured = false;  // per template instance
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsTotal);
    if (e != hipSuccess) return e;
    configured = true;
  }
  // two tile stages plus the block ids of one chunk (a chunk that does not start on a block boundary spans one more)
  const int blk_entries = (p.chunk_len >> p.block_shift) + 2;
  const int lds_bytes = kStages * kStageBytes + (blk_entries < kMaxChunkBlocks ? blk_entries : kMaxChunkBlocks) * 4;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * NW), lds_bytes, stream, p);
  return hipGetLastError();
}

template <int NW, int RB>
hipError_t launch_shape(const AttnParams &p, bool kv_fp8, bool br_fp8, hipStream_t stream) {
  if (kv_fp8 && br_fp8) return launch_variant<true, true, NW, RB>(p, stream);
  if (kv_fp8 && !br_fp8) return launch_variant<true, false, NW, RB>(p, stream);
  if (!kv_fp8 && !br_fp8) return launch_variant<false, false, NW, RB>(p, stream);
  return hipErrorInvalidValue;
}

// Kernel shapes: (wavefronts per workgroup, 32-row blocks per wavefront).
constexpr int kShapes[][2] = {{8, 1}, {4, 2}, {4, 1}};
constexpr int kNumShapes = 3;

}  // namespace

int attn_mfma_num_shapes() { return kNumShapes; }
int attn_mfma_tile_m(int shape) { return 32 * kShapes[shape][0] * kShapes[shape][1]; }
int attn_mfma_max_chunk_blocks() { return kMaxChunkBlocks; }

hipError_t launch_attn_mfma(const AttnParams &p, int shape, bool kv_fp8, bool br_fp8, hipStream_t stream) {
  ProfileScope scope(SLOT_ATTN_MFMA, stream);
  switch (shape) {
    case 0: return launch_shape<8, 1>(p, kv_fp8, br_fp8, stream);
    case 1: return launch_shape<4, 2>(p, kv_fp8, br_fp8, stream);
    case 2: return launch_shape<4, 1>(p, kv_fp8, br_fp8, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace la
