// Shared-prefix verify attention, bf16 MFMA path (gfx950).
//
// The verification pass expands all drafted branches against one shared prefix
// (Algorithm 1, "in parallel do"; prefixes x'_j).  Here the R = gamma*L*G query
// rows that share a KV head are tiled into row tiles; a workgroup owns
// (row tile, kv head, prefix chunk), streams the chunk's K/V tiles through LDS
// once and reuses every tile for all its rows.  The workgroup that owns the last
// chunk of a request also reduces the branch-private keys under the mask
// "same branch and key position <= query position" and, for nested branches
// (x'_j = x (+) s^_0 .. s^_{j-1}), the part of the request's drafted chain that each
// branch sees, or for a draft tree (W alternative steps per position) the pool tokens
// of the steps on each branch's root path.
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
#include <mutex>

#include "attn_common.hpp"

namespace la {
namespace {

constexpr int kD = 128;                      // head dim
constexpr int kTileN = 64;                   // keys per tile
constexpr int kKRow = kD * 2 + 16;           // bytes per key row of the K tile in LDS (padded)
constexpr int kVRow = kTileN * 2 + 16;       // bytes per d row of the V^T tile in LDS (padded)
constexpr int kKTileBytes = kTileN * kKRow;  // 17408
constexpr int kVTileBytes = kD * kVRow;      // 18432
constexpr int kStageBytes = kKTileBytes + kVTileBytes;
constexpr int kMaxChunkBlocks = 4096;        // block ids of one chunk kept in LDS
constexpr int kMaxStages = 3;
constexpr int kLdsTotal = kMaxStages * kStageBytes + kMaxChunkBlocks * 4;  // stages + block ids: 123904

// Where the keys of one tile come from.
struct TileSrc {
  const uint8_t *k_base, *v_base;  // prefix: cache base of this kv head; branch: row of token 0 of this request/head
  const int32_t *blk;              // prefix: physical block ids of this chunk (LDS), indexed from first_lb
  int first_lb;                    // prefix: logical block of blk[0]
  int first;                       // first key of the tile (prefix: token index; branch: token t = g*L+j)
  int limit;                       // keys >= limit are zero filled
};

// Staging registers of one K tile and one V tile per thread: 16-byte pieces of K rows; of V, four consecutive
// head-dim columns (4 bytes fp8, 8 bytes bf16) of the four keys of a key quad.
template <bool FP8, int NT>
struct TileRegs {
  static constexpr int kNK = (FP8 ? 512 : 1024) / NT;  // K pieces per thread
  static constexpr int kNV = 512 / NT;                 // V key quads per thread
  static constexpr int kVW = FP8 ? 1 : 2;              // dwords per key of a quad
  u32x4 k[kNK];
  uint32_t v[4 * kNV * kVW];
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
  constexpr int kVW = TileRegs<FP8, NT>::kVW;
#pragma unroll
  for (int e = 0; e < TileRegs<FP8, NT>::kNV; ++e) {
    const int idx = tid + NT * e;
    const int kq = idx >> 5;            // 32 pieces of four columns per key row
    const int piece = idx & 31;
    const int tok0 = s.first + 4 * kq;  // the four keys of a quad share a cache block (block_size % 16 == 0)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int tok = tok0 + c;
      const int tc = (FULL && PREFIX) ? tok : min(tok, s.limit - 1);
      const uint8_t *src = key_row<FP8, PREFIX>(p, s, s.v_base, tc) + piece * 4 * kVW;
#pragma unroll
      for (int w = 0; w < kVW; ++w) {
        const uint32_t val = *(const uint32_t *)(src + 4 * w);
        r.v[(4 * e + c) * kVW + w] = ((FULL && PREFIX) || tok < s.limit) ? val : 0u;
      }
    }
  }
}

// Full prefix tiles, the steady state: everything about an address that does not change from tile to tile is
// computed once per thread.  A tile starts at a multiple of 64 tokens and blocks hold a power of two >= 16 tokens, so
// for token first + tl (tl < 64 fixed per thread)
//   block index   = (first >> shift) + (tl >> shift)          (no carry between the two terms)
//   offset inside = (first & (bs-1)) + (tl & (bs-1))
// which leaves one LDS read of the block id and one 64-bit multiply-add per load.
template <bool FP8, int NT>
struct PrefixLoader {
  static constexpr int kNK = TileRegs<FP8, NT>::kNK, kNV = TileRegs<FP8, NT>::kNV, kVW = TileRegs<FP8, NT>::kVW;
  static constexpr int row_bytes = kD * (FP8 ? 1 : 2);
  const int32_t *blk;                        // LDS: block ids of the chunk
  int slot_k[kNK], slot_v[kNV];              // tl >> shift: block slot relative to the tile's first block
  const uint8_t *base_k[kNK], *base_v[kNV];  // cache base of the kv head + the thread's fixed byte offset
  size_t blk_stride;
  int shift, bs_mask, first_lb;

  __device__ __forceinline__ void init(const AttnParams &p, const TileSrc &s, int tid) {
    shift = p.block_shift;
    bs_mask = p.block_size - 1;
    first_lb = s.first_lb;
    blk = s.blk;
    blk_stride = ((size_t)p.Hkv << p.block_shift) * row_bytes;
    constexpr int k_piece_shift = FP8 ? 3 : 4;
#pragma unroll
    for (int e = 0; e < kNK; ++e) {
      const int idx = tid + NT * e;
      const int tl = idx >> k_piece_shift;
      slot_k[e] = tl >> shift;
      base_k[e] = s.k_base + (size_t)(tl & bs_mask) * row_bytes + (idx & ((1 << k_piece_shift) - 1)) * 16;
    }
#pragma unroll
    for (int e = 0; e < kNV; ++e) {
      const int idx = tid + NT * e;
      const int tl = 4 * (idx >> 5);
      slot_v[e] = tl >> shift;
      base_v[e] = s.v_base + (size_t)(tl & bs_mask) * row_bytes + (idx & 31) * 4 * kVW;
    }
  }
  // `first`: first token of the tile (a multiple of 64, every key of the tile valid)
  __device__ __forceinline__ void load(int first, TileRegs<FP8, NT> &r) const {
    const int rel = (first >> shift) - first_lb;
    const size_t inside = (size_t)(first & bs_mask) * row_bytes;
#pragma unroll
    for (int e = 0; e < kNK; ++e)
      r.k[e] = *(const u32x4 *)(base_k[e] + (size_t)(uint32_t)blk[rel + slot_k[e]] * blk_stride + inside);
#pragma unroll
    for (int e = 0; e < kNV; ++e) {
      const uint8_t *row = base_v[e] + (size_t)(uint32_t)blk[rel + slot_v[e]] * blk_stride + inside;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if constexpr (kVW == 1) {
          r.v[4 * e + c] = *(const uint32_t *)(row + c * row_bytes);
        } else {
          const u32x2 pair = *(const u32x2 *)(row + c * row_bytes);
          r.v[(4 * e + c) * 2] = pair[0];
          r.v[(4 * e + c) * 2 + 1] = pair[1];
        }
      }
    }
  }
};

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
      const int kq = idx >> 5;
      const int d0 = 4 * (idx & 31);
      // of key c: bf16 pairs (d0, d0+1) in v[2(4e+c)] and (d0+2, d0+3) in v[2(4e+c)+1]; columns d0..d0+3 live in
      // rows (d0/4) + 32*{0,1,2,3}: consecutive lanes write consecutive rows
      const uint32_t *lo = &r.v[8 * e], *hi = &r.v[8 * e + 1];  // stride 2 between keys
      uint8_t *dst = vt + (d0 >> 2) * kVRow + vt_pos(kq) * 2;
      *(u32x2 *)(dst) = u32x2{__builtin_amdgcn_perm(lo[2], lo[0], 0x05040100u),
                              __builtin_amdgcn_perm(lo[6], lo[4], 0x05040100u)};
      *(u32x2 *)(dst + 32 * kVRow) = u32x2{__builtin_amdgcn_perm(lo[2], lo[0], 0x07060302u),
                                           __builtin_amdgcn_perm(lo[6], lo[4], 0x07060302u)};
      *(u32x2 *)(dst + 64 * kVRow) = u32x2{__builtin_amdgcn_perm(hi[2], hi[0], 0x05040100u),
                                           __builtin_amdgcn_perm(hi[6], hi[4], 0x05040100u)};
      *(u32x2 *)(dst + 96 * kVRow) = u32x2{__builtin_amdgcn_perm(hi[2], hi[0], 0x07060302u),
                                           __builtin_amdgcn_perm(hi[6], hi[4], 0x07060302u)};
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


// One 64-key tile from an LDS stage, as two 32-key blocks whose MFMA and VALU work is interleaved:
//     S0 = K0 Q^T                    |
//     S1 = K1 Q^T                    |  P0 = 2^(S0 - m)          (VALU next to the MFMAs of the other block)
//     O += V0^T P0                   |  P1 = 2^(S1 - m)
//     O += V1^T P1                   |  tail()  (the caller's LDS stores of the next tile)
//   first / limit   MASK_TAIL: keys with first + key >= limit are masked
//                   MASK_BRANCH: key token first + key is visible to a row iff row_bstart <= token <= row_tok
//                   MASK_TREE: pool token first + key (< limit) is visible to a row iff its segment is in row_mask
//   crel            score scale of this key segment relative to the prefix scale that Q already carries (1 for prefix
//                   tiles); voff/lmul move a differently scaled V segment into the accumulator's units
//                   (p' = p * 2^voff, l += sum(p') * lmul)
//   k0              the K fragments of key block 0.  K0_READY: the caller already holds them (fetched while the
//                   previous tile was finishing); otherwise they are read here.  With next_kt != nullptr the block-0
//                   fragments of the tile staged at next_kt are fetched behind the last MFMAs and left in k0.
template <int RB, int MASK, bool K0_READY, bool PREFETCH, int GL = 0, typename Tail>
__device__ __forceinline__ void compute_tile(const uint8_t *kt, const uint8_t *next_kt, bf16x8 (&k0)[8],
                                             RowState<RB> &st, int ln, int lh, int first, int limit, float crel,
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
  // Full prefix tiles start S^T from -base (base == running maximum once one exists), so the MFMAs deliver s - m
  // and the probabilities need no multiply-add in front of the exponential, unless a maximum is raised in this
  // tile.  Other tiles (masked, or with their own score scale) start from zero and take the general form.
  constexpr bool kFastable = MASK == MASK_NONE;
  float binit[RB];
  f32x16 c_init[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    binit[rb] = kFastable ? st.base[rb] : 0.f;
    c_init[rb] = kFastable ? st.negb[rb] : zero;
  }
  auto exp_offset = [&](float (&off)[RB]) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      off[rb] = binit[rb] + voff - ((st.m_run[rb] == -INFINITY) ? 0.f : st.m_run[rb]);
  };

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
      s0[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0[t], st.qf[rb][t], t == 0 ? c_init[rb] : s0[rb], 0, 0, 0);
    k1[t] = load_k(t, 1);
  }
  // Order inside this stretch: the LDS addresses of the stage and, when the caller has just issued the global loads
  // of a later tile (GL > 0 load groups), the LDS reads of their block ids first; then one K1 fragment read behind
  // every MFMA, the 64-bit address arithmetic of the global loads once the block ids have arrived, and the loads.
  __builtin_amdgcn_sched_group_barrier(kSgSalu, 8, 0);
  __builtin_amdgcn_sched_group_barrier(kSgValu, 2 + 2 * GL, 0);
  __builtin_amdgcn_sched_group_barrier(kSgDsRead, GL, 0);
  if constexpr (!K0_READY) __builtin_amdgcn_sched_group_barrier(kSgDsRead, 8, 0);
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    __builtin_amdgcn_sched_group_barrier(kSgMfma, RB, 0);
    __builtin_amdgcn_sched_group_barrier(kSgDsRead, 1, 0);
    if (t == 1 && GL > 0) __builtin_amdgcn_sched_group_barrier(kSgValu, 5 * GL, 0);
    if (t == 2 && GL > 0) __builtin_amdgcn_sched_group_barrier(kSgVmemRead, 5 * GL, 0);
  }
  // ---- S1 = K1 Q^T next to P0, then O += V0^T P0 next to P1.  Full prefix tiles compute P = 2^x straight from the
  //      accumulators, without waiting for the block maximum; the maximum is formed beside it and, in the rare case
  //      that a row's maximum has to be raised, P of that block is computed again in the general form.  The V
  //      fragments are fetched from LDS behind the MFMAs.
  uint32_t p0[RB][8], p1[RB][8];
  float sum0[RB], sum1[RB], mt[RB], alpha[RB], off[RB];
  bf16x8 v0[2][4], v1[2][4];
#pragma unroll
  for (int t = 0; t < 8; ++t)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      s1[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1[t], st.qf[rb][t], t == 0 ? c_init[rb] : s1[rb], 0, 0, 0);
  mask_block<RB, MASK>(s0, st, 0, lh, first, limit);
  if constexpr (kFastable) block_probs<RB, true>(s0, crel, off, p0, sum0);
  block_max<RB>(s0, crel, binit, mt);
  // V fragments are fetched half a block ahead of the MFMAs that use them (16 registers in flight, not 32)
#pragma unroll
  for (int db = 0; db < 4; ++db) v0[0][db] = load_v(db, 0, 0);
#pragma unroll
  for (int i = 0; i < 8; ++i) {  // per step: RB MFMAs, a share of the VALU work, one LDS read
    __builtin_amdgcn_sched_group_barrier(kSgMfma, RB, 0);
    __builtin_amdgcn_sched_group_barrier(kSgValu, 6 * RB, 0);
    __builtin_amdgcn_sched_group_barrier(kSgDsRead, 1, 0);
  }
  // keep the speculative probabilities on this side of the branch below (otherwise they are sunk into the arm that
  // uses them and no longer overlap the MFMAs above)
  if constexpr (kFastable) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      asm volatile("" ::"v"(p0[rb][0]), "v"(p0[rb][1]), "v"(p0[rb][2]), "v"(p0[rb][3]), "v"(p0[rb][4]),
                   "v"(p0[rb][5]), "v"(p0[rb][6]), "v"(p0[rb][7]), "v"(sum0[rb]));
  }
  const bool raise0 = raise_max<RB>(mt, st, alpha);
  if (!kFastable || raise0) {
    if (raise0) rescale<RB>(st, alpha);
    exp_offset(off);
    block_probs<RB, false>(s0, crel, off, p0, sum0);
  }
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) st.l_run[rb] += sum0[rb] * lmul;

#pragma unroll
  for (int db = 0; db < 4; ++db) v0[1][db] = load_v(db, 0, 1);
  __builtin_amdgcn_sched_group_barrier(kSgDsRead, 4, 0);
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
  mask_block<RB, MASK>(s1, st, 1, lh, first, limit);
  if constexpr (kFastable) block_probs<RB, true>(s1, crel, off, p1, sum1);
  block_max<RB>(s1, crel, binit, mt);
#pragma unroll
  for (int db = 0; db < 4; ++db) v1[0][db] = load_v(db, 1, 0);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    __builtin_amdgcn_sched_group_barrier(kSgMfma, RB, 0);
    __builtin_amdgcn_sched_group_barrier(kSgValu, 6 * RB, 0);
    __builtin_amdgcn_sched_group_barrier(kSgDsRead, 1, 0);
  }
  if constexpr (kFastable) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      asm volatile("" ::"v"(p1[rb][0]), "v"(p1[rb][1]), "v"(p1[rb][2]), "v"(p1[rb][3]), "v"(p1[rb][4]),
                   "v"(p1[rb][5]), "v"(p1[rb][6]), "v"(p1[rb][7]), "v"(sum1[rb]));
  }
  const bool raise1 = raise_max<RB>(mt, st, alpha);  // the accumulators now hold block 0 in the old units
  if (!kFastable || raise0 || raise1) {  // after a raise in block 0, S1 is no longer relative to the maximum
    if (raise1) rescale<RB>(st, alpha);
    exp_offset(off);
    block_probs<RB, false>(s1, crel, off, p1, sum1);
  }
  if (raise0 || raise1) {  // keep base == running maximum for the next tile
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float bnew = (st.m_run[rb] == -INFINITY) ? 0.f : st.m_run[rb];
      st.base[rb] = bnew;
#pragma unroll
      for (int j = 0; j < 16; ++j) st.negb[rb][j] = -bnew;
    }
  }
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) st.l_run[rb] += sum1[rb] * lmul;

  // ---- O += V1^T P1 next to the caller's tail work ----------------------------------------------
#pragma unroll
  for (int db = 0; db < 4; ++db) v1[1][db] = load_v(db, 1, 1);
  __builtin_amdgcn_sched_group_barrier(kSgDsRead, 4, 0);
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

// NW wavefronts of RB 32-row blocks each: a row tile of 32*NW*RB rows.  STAGES LDS stages per workgroup:
//   3: tile i is computed on while tile i+1 is resident (its first K fragments are fetched early) and tile i+2 is
//      written; one workgroup per CU.  The shape for large row counts, where the matrix cores are the limit.
//   2: tile i is computed on while tile i+1 is written and tiles i+2, i+3 are in flight from HBM; two workgroups
//      share a CU, which hides the start-up and per-tile latencies when the row count is small and the KV
//      stream is the limit.
//   EXTRA: 0 = flat call, 1 = the call carries a drafted chain (nested form), 2 = a pool of drafted tokens with
//   segment masks (tree form).  A build switch rather than a run-time test so that the flat kernels keep the
//   register allocation they were tuned with.
template <bool KV_FP8, bool BR_FP8, int NW, int RB, int STAGES, int EXTRA>
__global__ __launch_bounds__(64 * NW, (NW * RB <= 4) ? 2 : 1) void attn_mfma_kernel(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  constexpr int NT = 64 * NW;
  constexpr int kTileM = 32 * NW * RB;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
  // workgroups are dispatched in blockIdx order: the last chunk, which also carries the chain and branch-private
  // tiles and so runs longest, goes first instead of into the tail of the launch
  c = n_chunks - 1 - c;
  int k_begin, k_end;
  attn_chunk_range(P, p.chunk_len, p.last_short, c, &k_begin, &k_end);
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
  int32_t *blk_lds = (int32_t *)(lds + STAGES * kStageBytes);
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

  // two-stage shape: a wavefront whose rows all lie past R stages tiles but computes nothing
  const bool active = STAGES == 3 || r0 + wave * RB * 32 < p.R;

  // Score scales of the two key segments, in log2 units.  Q is multiplied by the prefix scale when it is loaded
  // (and rounded to bf16 again), so prefix scores leave the MFMAs ready for the exponential; a branch segment with
  // another scale is corrected by crel_branch.
  float c_prefix = p.scale_log2, crel_branch = 1.0f;
  float vmul_branch = 1.0f;  // branch V is multiplied by this to live in the prefix segment's V units
  float v_out = 1.0f;
  if (KV_FP8) {
    const float ks = p.k_scale ? p.k_scale[kvh] : 1.0f;
    const float vs = p.v_scale ? p.v_scale[kvh] : 1.0f;
    c_prefix *= ks;
    v_out = vs;
    if (!BR_FP8) {
      crel_branch = 1.0f / ks;
      vmul_branch = 1.0f / vs;
    }
  }
  const float voff_branch = __builtin_log2f(vmul_branch);
  const float lmul_branch = 1.0f / vmul_branch;

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
#pragma unroll
      for (int w = 0; w < 4; ++w) {  // bf16 pair -> fp32, times the prefix scale, back to bf16 (round to nearest even)
        const uint32_t word = v[w];
        const uint32_t wl = word << 16, wh = word & 0xffff0000u;
        v[w] = pack_bf16(__builtin_bit_cast(float, wl) * c_prefix, __builtin_bit_cast(float, wh) * c_prefix);
      }
      st.qf[rb][t] = __builtin_bit_cast(bf16x8, v);
    }
    st.m_run[rb] = -INFINITY;
    st.l_run[rb] = 0.f;
    st.base[rb] = 0.f;
#pragma unroll
    for (int j = 0; j < 16; ++j) st.negb[rb][j] = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int j = 0; j < 16; ++j) st.o[db][rb][j] = 0.f;
  }

  __syncthreads();  // block ids visible

  // ---- phase 1: the unmasked prefix tiles -----------------------------------------------------
  bf16x8 k0[8];
  if constexpr (STAGES == 3) {
    // ring of three stages.  iteration i: global loads of tile i+2 are in flight, tile i is computed from stage
    // i%3 (its block-0 K fragments were fetched while tile i-1 finished), the block-0 fragments of tile i+1 are
    // fetched from stage (i+1)%3, and tile i+2 is written to stage (i+2)%3, which every wavefront stopped
    // reading at the barrier before.
    if (n_full > 0) {
      TileRegs<KV_FP8, NT> regs;
      PrefixLoader<KV_FP8, NT> loader;
      loader.init(p, pre, tid);
      auto gload = [&](int it) { loader.load(k_begin + it * kTileN, regs); };
      // byte offsets of the stages holding tile it, it+1 and it+2; rotated once per tile
      int o_cur = 0, o_next = kStageBytes, o_store = 2 * kStageBytes;
      gload(0);
      tile_store<KV_FP8, NT>(lds + o_cur, tid, regs);
      if (n_full > 1) {
        gload(1);
        tile_store<KV_FP8, NT>(lds + o_next, tid, regs);
      }
      __syncthreads();
      {
        const uint8_t *krow = lds + ln * kKRow + lh * 16;
#pragma unroll
        for (int t = 0; t < 8; ++t) k0[t] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(krow + t * 32));
      }
      int it = 0;
      for (; it + 2 < n_full; ++it) {  // steady state: nothing conditional
        gload(it + 2);
        compute_tile<RB, MASK_NONE, true, true, TileRegs<KV_FP8, NT>::kNK + TileRegs<KV_FP8, NT>::kNV>(
            lds + o_cur, lds + o_next, k0, st, ln, lh, 0, 0, 1.f, 0.f, 1.f,
            [&] { tile_store<KV_FP8, NT>(lds + o_store, tid, regs); });
        __syncthreads();
        const int o = o_cur;
        o_cur = o_next;
        o_next = o_store;
        o_store = o;
      }
      if (it + 1 < n_full) {  // second to last tile: nothing left to load
        compute_tile<RB, MASK_NONE, true, true>(lds + o_cur, lds + o_next, k0, st, ln, lh, 0, 0, 1.f, 0.f, 1.f, [] {});
        o_cur = o_next;
      }
      compute_tile<RB, MASK_NONE, true, false>(lds + o_cur, nullptr, k0, st, ln, lh, 0, 0, 1.f, 0.f, 1.f, [] {});
      __syncthreads();
    }
  } else {
    // two stages, one register set.  Iteration i computes on stage i%2 and then writes tile i+1 (loaded during
    // iteration i-1) to the other stage and issues the loads of tile i+2.  Those loads have one tile time to
    // arrive, less than an HBM round trip under load, so every 128-byte line of a tile is touched four tiles
    // ahead with a one-word load whose value is only folded into a sink: the staging loads then hit L2.
    uint32_t sink = 0;
    if (n_full > 0) {
      TileRegs<KV_FP8, NT> regs;
      PrefixLoader<KV_FP8, NT> loader;
      loader.init(p, pre, tid);
      auto gload = [&](int it) { loader.load(k_begin + it * kTileN, regs); };
      constexpr int kLinesPerRow = kv_row / 128;       // 1 (fp8) or 2 (bf16)
      constexpr int kLines = kTileN * kLinesPerRow;    // lines of the K tile; the V tile has as many
      static_assert(2 * kLines <= NT, "one touch per thread");
      auto touch = [&](int it) -> uint32_t {
        if (it >= n_full || tid >= 2 * kLines) return 0u;
        pre.first = k_begin + it * kTileN;
        const int line = tid % kLines;
        const uint8_t *base = tid < kLines ? pre.k_base : pre.v_base;
        return *(const uint32_t *)(key_row<KV_FP8, true>(p, pre, base, pre.first + line / kLinesPerRow) +
                                   (line % kLinesPerRow) * 128);
      };
      const uint32_t t1 = touch(1), t2 = touch(2), t3 = touch(3);
      gload(0);
      tile_store<KV_FP8, NT>(lds, tid, regs);
      if (n_full > 1) gload(1);
      uint32_t pf = t1 ^ t2 ^ t3;
      __syncthreads();
      for (int it = 0; it < n_full; ++it) {
        const uint8_t *cur = lds + (it & 1) * kStageBytes;
        uint8_t *other = lds + ((it + 1) & 1) * kStageBytes;
        auto tail = [&] {
          if (it + 1 < n_full) {
            tile_store<KV_FP8, NT>(other, tid, regs);
            if (it + 2 < n_full) gload(it + 2);
          }
          sink ^= pf;
          pf = touch(it + 4);
        };
        if (active)
          compute_tile<RB, MASK_NONE, false, false>(cur, nullptr, k0, st, ln, lh, 0, 0, 1.f, 0.f, 1.f, tail);
        else
          tail();
        __syncthreads();
      }
      sink ^= pf;
    }
    // never true (R >= 1): keeps the touched words alive without a store on any real path
    if (p.R < 0) p.part_ml[0] = __builtin_bit_cast(float, sink);
  }
  // ---- phase 2: the partly filled prefix tile -------------------------------------------------
  if (has_tail) {
    TileRegs<KV_FP8, NT> regs;
    pre.first = k_begin + n_full * kTileN;
    tile_load<KV_FP8, true, false, NT>(p, pre, tid, regs);
    tile_store<KV_FP8, NT>(lds, tid, regs);
    __syncthreads();
    if (active)
      compute_tile<RB, MASK_TAIL, false, false>(lds, nullptr, k0, st, ln, lh, pre.first, k_end, 1.f, 0.f, 1.f,
                                                [] {});
    __syncthreads();
  }
  // ---- phase 3 (tree form): the pool of drafted tokens under the segment masks (last chunk only) ----------------
  if constexpr (EXTRA == 2) {
    if (c == n_chunks - 1) {
      uint64_t seen_any = 0;  // wavefront-uniform: segments seen by any branch of this row tile
      for (int g = t_lo / p.L; g <= t_hi / p.L; ++g) seen_any |= p.seg_mask[b * p.gamma + g];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) st.row_mask[rb] = p.seg_mask[b * p.gamma + st.row_tok[rb] / p.L];
      TileSrc pool = brs;
      const size_t pool_off = ((size_t)b * p.C * p.Hkv + kvh) * br_row;
      pool.k_base = (const uint8_t *)p.k_chain + pool_off;
      pool.v_base = (const uint8_t *)p.v_chain + pool_off;
      pool.limit = p.C;
      for (int first = 0; first < p.C; first += kTileN) {
        // lane k of every wavefront: segment of pool token first + k.  A tile none of whose tokens any branch of
        // the row tile sees is skipped (the same decision in every wavefront: same data).
        const int tok = first + lane;
        const int seg = p.pool_seg[(size_t)b * p.C + min(tok, p.C - 1)];
        st.tile_seg = seg;
        if (__builtin_amdgcn_ballot_w64(tok < p.C && ((seen_any >> seg) & 1)) == 0) continue;
        TileRegs<BR_FP8, NT> regs;
        pool.first = first;
        tile_load<BR_FP8, false, false, NT>(p, pool, tid, regs);
        tile_store<BR_FP8, NT>(lds, tid, regs);
        __syncthreads();
        if (active)
          compute_tile<RB, MASK_TREE, false, false>(lds, nullptr, k0, st, ln, lh, first, p.C, crel_branch, voff_branch,
                                                    lmul_branch, [] {});
        __syncthreads();
      }
    }
  }
  // ---- phase 3: the drafted chain of a nested problem, then the branch-private tiles (last chunk only) ----------
  // Branch g sees chain tokens 0 .. vis[g]-1: that is the branch mask with the window [0, vis-1], so the rows'
  // windows are swapped for it while the chain tiles run and both segments share one loop.
  int n_chain = 0;
  TileSrc chn = brs;
  if (EXTRA == 1 && c == n_chunks - 1) {
    int vmax = 0;  // wavefront-uniform: the longest visible part among the branches of this row tile
    for (int g = t_lo / p.L; g <= t_hi / p.L; ++g) vmax = max(vmax, p.chain_vis[b * p.gamma + g]);
    vmax = min(vmax, p.C);
    n_chain = (vmax + kTileN - 1) / kTileN;
    const size_t ch_off = ((size_t)b * p.C * p.Hkv + kvh) * br_row;
    chn.k_base = (const uint8_t *)p.k_chain + ch_off;
    chn.v_base = (const uint8_t *)p.v_chain + ch_off;
    chn.limit = vmax;
    if (n_chain > 0) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        st.row_tok[rb] = p.chain_vis[b * p.gamma + st.row_tok[rb] / p.L] - 1;
        st.row_bstart[rb] = 0;
      }
    }
  }
  // the loads of tile it+1 are in flight while tile it is computed on
  TileRegs<BR_FP8, NT> bregs;
  auto load_extra = [&](int it) {
    TileSrc src = it < n_chain ? chn : brs;
    src.first = it < n_chain ? it * kTileN : tk0 + (it - n_chain) * kTileN;
    tile_load<BR_FP8, false, false, NT>(p, src, tid, bregs);
    return src.first;
  };
  int first_cur = n_chain + n_priv > 0 ? load_extra(0) : 0;
  for (int it = 0; it < n_chain + n_priv; ++it) {
    if (EXTRA == 1 && it == n_chain && n_chain > 0) {  // back to the rows' own windows
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        st.row_tok[rb] = min(row[rb], p.R - 1) / p.G;
        st.row_bstart[rb] = (st.row_tok[rb] / p.L) * p.L;
      }
    }
    tile_store<BR_FP8, NT>(lds, tid, bregs);
    __syncthreads();
    const int first = first_cur;
    if (it + 1 < n_chain + n_priv) first_cur = load_extra(it + 1);
    if (active)
      compute_tile<RB, MASK_BRANCH, false, false>(lds, nullptr, k0, st, ln, lh, first, 0, crel_branch, voff_branch,
                                                  lmul_branch, [] {});
    __syncthreads();
  }
  if (EXTRA == 1 && n_chain > 0 && n_priv == 0) {  // not reached (the last chunk always has private tiles); keeps row_tok honest
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) st.row_tok[rb] = min(row[rb], p.R - 1) / p.G;
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

template <bool KV_FP8, bool BR_FP8, int NW, int RB, int STAGES, int EXTRA>
hipError_t launch_variant(const AttnParams &p, hipStream_t stream) {
  const int grid = p.Hkv * p.n_row_tiles * p.total_units;
  auto kern = attn_mfma_kernel<KV_FP8, BR_FP8, NW, RB, STAGES, EXTRA>;
  static std::once_flag once;  // per template instance
  static hipError_t configured = hipSuccess;
  std::call_once(once, [&] {
    configured = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsTotal);
  });
  if (configured != hipSuccess) return configured;
  // the tile stages plus the block ids of one chunk (a chunk that does not start on a block boundary spans one more)
  const int blk_entries = (attn_max_chunk_tokens(p.chunk_len, p.last_short) >> p.block_shift) + 2;
  const int lds_bytes = STAGES * kStageBytes + (blk_entries < kMaxChunkBlocks ? blk_entries : kMaxChunkBlocks) * 4;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * NW), lds_bytes, stream, p);
  return hipGetLastError();
}

template <int NW, int RB, int STAGES>
hipError_t launch_shape(const AttnParams &p, bool kv_fp8, bool br_fp8, hipStream_t stream) {
  if (p.C > 0 && p.pool_seg) {
    if (kv_fp8 && br_fp8) return launch_variant<true, true, NW, RB, STAGES, 2>(p, stream);
    if (kv_fp8 && !br_fp8) return launch_variant<true, false, NW, RB, STAGES, 2>(p, stream);
    if (!kv_fp8 && !br_fp8) return launch_variant<false, false, NW, RB, STAGES, 2>(p, stream);
    return hipErrorInvalidValue;
  }
  if (p.C > 0) {
    if (kv_fp8 && br_fp8) return launch_variant<true, true, NW, RB, STAGES, 1>(p, stream);
    if (kv_fp8 && !br_fp8) return launch_variant<true, false, NW, RB, STAGES, 1>(p, stream);
    if (!kv_fp8 && !br_fp8) return launch_variant<false, false, NW, RB, STAGES, 1>(p, stream);
    return hipErrorInvalidValue;
  }
  if (kv_fp8 && br_fp8) return launch_variant<true, true, NW, RB, STAGES, 0>(p, stream);
  if (kv_fp8 && !br_fp8) return launch_variant<true, false, NW, RB, STAGES, 0>(p, stream);
  if (!kv_fp8 && !br_fp8) return launch_variant<false, false, NW, RB, STAGES, 0>(p, stream);
  return hipErrorInvalidValue;
}

// Kernel shapes: (wavefronts per workgroup, 32-row blocks per wavefront, LDS stages).
constexpr int kShapes[][3] = {{8, 1, 3}, {4, 1, 2}};
constexpr int kNumShapes = 2;

}  // namespace

int attn_mfma_num_shapes() { return kNumShapes; }
int attn_mfma_tile_m(int shape) { return 32 * kShapes[shape][0] * kShapes[shape][1]; }
int attn_mfma_wgs_per_cu(int shape) { return kShapes[shape][2] == 2 ? 2 : 1; }
int attn_mfma_max_chunk_blocks() { return kMaxChunkBlocks; }

hipError_t launch_attn_mfma(const AttnParams &p, int shape, bool kv_fp8, bool br_fp8, hipStream_t stream) {
  ProfileScope scope(SLOT_ATTN_MFMA, stream);
  switch (shape) {
    case 0: return launch_shape<8, 1, 3>(p, kv_fp8, br_fp8, stream);
    case 1: return launch_shape<4, 1, 2>(p, kv_fp8, br_fp8, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace la
