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
//                    4*m + db, so that consecutive lanes of the transposing writes hit
//                    consecutive rows and the four db accumulators of a lane are
//                    adjacent columns; fragment reads and staging writes are bank-conflict
//                    free, see v_piece_of and k_chunk_at),
//                    B = P^T (registers, bf16)
// Everything is kept in log2 units: p = 2^(s*c - m).
#include <mutex>
#include <type_traits>
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
constexpr int kMaxStages = 4;
constexpr int kLdsTotal = kMaxStages * kStageBytes + kMaxChunkBlocks * 4;  // stages + block ids: 159744
static_assert(kLdsTotal <= 160 * 1024, "LDS of one CU");

// Where the keys of one tile come from.
struct TileSrc {
  const uint8_t *k_base, *v_base;  // prefix: cache base of this kv head; branch: row of token 0 of this request/head
  const int32_t *blk;              // prefix: physical block ids of this chunk (LDS), indexed from first_lb
  int first_lb;                    // prefix: logical block of blk[0]
  int first;                       // first key of the tile (prefix: token index; branch: token t = g*L+j)
  int limit;                       // keys >= limit are zero filled
};

// With an fp8 cache, K rows in LDS hold their sixteen 16-byte chunks (eight head-dim columns each) in the order even
// chunks, odd chunks: position q holds chunk k_chunk_at(q).  A thread staging an fp8 row piece owns chunks 2p and 2p+1, and its two 16-byte
// stores go to positions p and 8 + p: eight consecutive lanes then write 128 contiguous bytes, which is what the LDS
// takes per cycle (at positions 2p and 2p + 1 lanes p and p + 4 met on the same banks).  The contraction runs over the
// head dimension, so the order is free as long as Q's fragments follow it (they are loaded in the same order).
__device__ __forceinline__ constexpr int k_chunk_at(int q) { return ((q & 7) << 1) | (q >> 3); }

// Which V piece a staging thread owns: key quad kq (keys 4kq .. 4kq+3) and column quad `piece` (columns 4 piece ..
// +3) of element idx = tid + NT*e.  The transposing LDS stores write eight bytes per lane to row `piece` (+ a
// constant) at the quad's place in the row.  LDS writes are served 128 bytes (16 lanes of eight bytes) per cycle over
// 32 four-byte banks, and at the 144-byte row pitch row r+8 falls on the banks of row r: 16 lanes cover the banks
// exactly when they are 8 consecutive rows times the two halves of a 16-byte chunk (key quads kq and kq ^ 2).
// (Measured with an in-bounds probe: 16 consecutive rows per 16 lanes take 8 cycles per store, this order 4.)
__device__ __forceinline__ void v_piece_of(int idx, int &kq, int &piece) {
  piece = (idx & 7) | (((idx >> 4) & 3) << 3);
  kq = (((idx >> 3) & 1) << 1) | ((idx >> 6) & 1) | ((idx >> 7) << 2);
}

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
//   KPERM (bf16 tiles): the tile goes to LDS in the chunk order of fp8 tiles (k_chunk_at), because it shares Q's
//   fragments with an fp8 cache; a thread then fetches the chunk of the LDS position it writes.
template <bool FP8, bool PREFIX, bool FULL, int NT, bool KPERM = false>
__device__ __forceinline__ void tile_load(const AttnParams &p, const TileSrc &s, int tid, TileRegs<FP8, NT> &r) {
  constexpr int k_piece_shift = FP8 ? 3 : 4;  // 16-byte pieces per key row: 8 (fp8) or 16 (bf16)
#pragma unroll
  for (int e = 0; e < TileRegs<FP8, NT>::kNK; ++e) {
    const int idx = tid + NT * e;
    const int tok = s.first + (idx >> k_piece_shift);
    const int tc = FULL ? tok : min(tok, s.limit - 1);
    const int piece = idx & ((1 << k_piece_shift) - 1);
    u32x4 val =
        *(const u32x4 *)(key_row<FP8, PREFIX>(p, s, s.k_base, tc) + ((FP8 || !KPERM) ? piece : k_chunk_at(piece)) * 16);
    if (!FULL && tok >= s.limit) val = u32x4{0, 0, 0, 0};
    r.k[e] = val;
  }
  constexpr int kVW = TileRegs<FP8, NT>::kVW;
#pragma unroll
  for (int e = 0; e < TileRegs<FP8, NT>::kNV; ++e) {
    const int idx = tid + NT * e;
    int kq, piece;                      // 32 pieces of four columns per key row
    v_piece_of(idx, kq, piece);
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
      int kq, piece;
      v_piece_of(idx, kq, piece);
      const int tl = 4 * kq;
      slot_v[e] = tl >> shift;
      base_v[e] = s.v_base + (size_t)(tl & bs_mask) * row_bytes + piece * 4 * kVW;
    }
  }
  // `first`: first token of the tile (a multiple of 64, every key of the tile valid)
  __device__ __forceinline__ void load(int first, TileRegs<FP8, NT> &r) const {
    int ids[kNK + kNV];
    fetch_ids(first, ids);
    load_k(first, ids, r);
    load_v(first, ids, r);
  }
  // The same in three steps, for a caller that spreads them between other work: the block ids from LDS, then the K
  // loads, then the V loads.
  __device__ __forceinline__ void fetch_ids(int first, int (&ids)[kNK + kNV]) const {
    const int rel = (first >> shift) - first_lb;
#pragma unroll
    for (int e = 0; e < kNK; ++e) ids[e] = blk[rel + slot_k[e]];
#pragma unroll
    for (int e = 0; e < kNV; ++e) ids[kNK + e] = blk[rel + slot_v[e]];
  }
  __device__ __forceinline__ void load_k(int first, const int (&ids)[kNK + kNV], TileRegs<FP8, NT> &r) const {
    const size_t inside = (size_t)(first & bs_mask) * row_bytes;
#pragma unroll
    for (int e = 0; e < kNK; ++e)
      r.k[e] = *(const u32x4 *)(base_k[e] + (size_t)(uint32_t)ids[e] * blk_stride + inside);
  }
  __device__ __forceinline__ void load_v(int first, const int (&ids)[kNK + kNV], TileRegs<FP8, NT> &r) const {
    const size_t inside = (size_t)(first & bs_mask) * row_bytes;
#pragma unroll
    for (int e = 0; e < kNV; ++e) {
      const uint8_t *row = base_v[e] + (size_t)(uint32_t)ids[kNK + e] * blk_stride + inside;
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
// bf16 on the way (exact: every e4m3 value is a bf16 value).  In three pieces (K; V columns d0, d0+1; V columns d0+2,
// d0+3) so that a caller can spread them between other work.
template <bool FP8, int NT>
__device__ __forceinline__ void tile_store_k(uint8_t *stage, int tid, const TileRegs<FP8, NT> &r) {
  uint8_t *kt = stage;
#pragma unroll
  for (int e = 0; e < TileRegs<FP8, NT>::kNK; ++e) {
    const int idx = tid + NT * e;
    if constexpr (!FP8) {
      *(u32x4 *)(kt + (idx >> 4) * kKRow + (idx & 15) * 16) = r.k[e];
    } else {
      uint32_t out[8];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t word = r.k[e][w];
        out[2 * w] = fp8x2_to_bf16x2<false>(word);
        out[2 * w + 1] = fp8x2_to_bf16x2<true>(word);
      }
      uint8_t *dst = kt + (idx >> 3) * kKRow + (idx & 7) * 16;  // chunks 2p, 2p+1 -> positions p, 8 + p
      *(u32x4 *)(dst) = u32x4{out[0], out[1], out[2], out[3]};
      *(u32x4 *)(dst + 128) = u32x4{out[4], out[5], out[6], out[7]};
    }
  }
}
// HALF 0: head-dim columns d0, d0+1 of the thread's four keys; HALF 1: columns d0+2, d0+3
template <bool FP8, int NT, int HALF>
__device__ __forceinline__ void tile_store_v(uint8_t *stage, int tid, const TileRegs<FP8, NT> &r) {
  uint8_t *vt = stage + kKTileBytes;
#pragma unroll
  for (int e = 0; e < TileRegs<FP8, NT>::kNV; ++e) {
    const int idx = tid + NT * e;
    int kq, piece;
    v_piece_of(idx, kq, piece);
    const int d0 = 4 * piece;
    // of key c: the bf16 pair (d0 + 2 HALF, d0 + 2 HALF + 1).  Columns d0..d0+3 live in rows (d0/4) + 32*{0,1,2,3}:
    // consecutive lanes write consecutive rows
    uint32_t w[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if constexpr (FP8)
        w[c] = fp8x2_to_bf16x2<HALF != 0>(r.v[4 * e + c]);
      else
        w[c] = r.v[8 * e + 2 * c + HALF];
    }
    uint8_t *dst = vt + ((d0 >> 2) + 64 * HALF) * kVRow + vt_pos(kq) * 2;
    *(u32x2 *)(dst) = u32x2{__builtin_amdgcn_perm(w[1], w[0], 0x05040100u), __builtin_amdgcn_perm(w[3], w[2], 0x05040100u)};
    *(u32x2 *)(dst + 32 * kVRow) =
        u32x2{__builtin_amdgcn_perm(w[1], w[0], 0x07060302u), __builtin_amdgcn_perm(w[3], w[2], 0x07060302u)};
  }
}
template <bool FP8, int NT>
__device__ __forceinline__ void tile_store(uint8_t *stage, int tid, const TileRegs<FP8, NT> &r) {
  tile_store_k<FP8, NT>(stage, tid, r);
  tile_store_v<FP8, NT, 0>(stage, tid, r);
  tile_store_v<FP8, NT, 1>(stage, tid, r);
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

// ---- block-pipelined steady state (four LDS stages, one 32-row block per wavefront) ----------------------------
// The full prefix tiles of a chunk are reduced as a stream of 32-key blocks b = 0, 1, 2, ... in a three-deep software
// pipeline: in slot b the MFMAs of S^T_{b+1} = K_{b+1} Q^T and of O^T += V_{b-1}^T P_{b-1}^T run while the VALU turns
// S^T_b into P^T_b.  Every slot therefore carries 16 MFMAs and one block's worth of exponentials, at every point of
// the loop, instead of MFMA-only and VALU-heavy stretches taking turns: a wavefront issues roughly one instruction
// per seven cycles, so the two wavefronts of a SIMD keep the matrix pipe busy only if neither of them ever has long
// runs of one kind.  The price is a fourth LDS stage (the V rows of the previous tile's second block are still read
// while the tile after next is written) and that the block maximum is not known when P is formed: P is computed as
// 2^(s - base) against the base the S^T accumulators were started from; the row sum doubles as the overflow guard (a
// sum above kTrigger sends the wavefront through the general form, which finds the true maximum and moves the base).
constexpr float kTrigger = 1024.0f;
constexpr int kAhead = 3;  // LDS fragment reads run this many MFMAs of their kind ahead of their use

struct PipeCarry {
  f32x16 s0[1];      // S^T of key block 0 of the tile about to be reduced (its MFMAs ran during the previous tile)
  float bs0;         // the base s0 was started from
  uint64_t stale0;   // all ones or zero (a lane mask, so that it stays in scalar registers): the base has moved since
                     // s0 was started, or there is none yet
  uint32_t pq[1][8]; // P^T of key block 1 of the previous tile, not yet multiplied into O (zero before the first)
  bf16x8 kf[kAhead]; // the first K fragments of the block whose S^T runs in the next slot
  bf16x8 vf[kAhead]; // the first V^T fragments of the block that is multiplied into O in the next slot
};

// One slot.  hook(i), i = 0..15, is called once per MFMA.  kS: the lane's K row of the block whose S^T accumulates (fragment t lies 32t bytes on); vP: the lane's
// V^T row of the block multiplied into O (fragment (db, t2) at db*32*kVRow + 32*t2); kS_next / vP_next: the same for
// the next slot, whose fragments 0..3 are left in kf / vf.  sc: the complete S^T (relative to its base) of the block
// in between; its probabilities go to pc (bf16 pairs), their fp32 sum to acc.
template <bool DO_S, bool NEXT_K, bool NEXT_V, int PRIO, typename Hook>
__device__ __forceinline__ void pipe_slot(const uint8_t *kS, const uint8_t *vP, const uint8_t *kS_next,
                                          const uint8_t *vP_next, bf16x8 (&kf)[kAhead], bf16x8 (&vf)[kAhead],
                                          const bf16x8 (&qf)[8], const f32x16 &c_init, f32x16 &s_new,
                                          const f32x16 &sc, const uint32_t (&pp)[8], f32x16 (&o)[4][1],
                                          uint32_t (&pc)[8], float &acc, Hook &&hook) {
  // fragment windows: entries 0..7 belong to this slot (0..kAhead-1 arrive in kf / vf), 8.. to the next one; the
  // fragment kAhead places further on is read behind every MFMA
  bf16x8 ka[8 + kAhead], va[8 + kAhead];
#pragma unroll
  for (int j = 0; j < kAhead; ++j) ka[j] = kf[j], va[j] = vf[j];
  float e_prev = 0.f, sum = 0.f;
  const u32x4 pw0 = {pp[0], pp[1], pp[2], pp[3]}, pw1 = {pp[4], pp[5], pp[6], pp[7]};
  const bf16x8 pf0 = __builtin_bit_cast(bf16x8, pw0), pf1 = __builtin_bit_cast(bf16x8, pw1);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int t = i >> 1, n = t + kAhead;
    // Issue priority falls with progress through the tile (3, 2 in slot A; 1, 0 in slot B): of the two wavefronts of a
    // SIMD the one that is behind wins the arbitration, so they stay within a quarter of a tile of each other and
    // neither is left to finish alone before the barrier (a lone wavefront keeps the matrix pipe only half busy).
    if (i == 0) __builtin_amdgcn_s_setprio(PRIO);
    if (i == 8) __builtin_amdgcn_s_setprio(PRIO - 1);
    if ((i & 1) == 0) {
      if constexpr (DO_S)
        s_new = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t], qf[t], t == 0 ? c_init : s_new, 0, 0, 0);
      if (n < 8) {
        if constexpr (DO_S) ka[n] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(kS + n * 32));
      } else {
        if constexpr (NEXT_K) ka[n] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(kS_next + (n - 8) * 32));
      }
    } else {
      // V^T fragment u: head-dim block u % 4, keys 16 (u / 4) .. +16 of the block
      o[t & 3][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[t], t < 4 ? pf0 : pf1, o[t & 3][0], 0, 0, 0);
      if (n < 8) {
        va[n] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(vP + (n & 3) * 32 * kVRow + (n >> 2) * 32));
      } else {
        if constexpr (NEXT_V)
          va[n] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(vP_next + ((n - 8) & 3) * 32 * kVRow + ((n - 8) >> 2) * 32));
      }
    }
    const float e = __builtin_amdgcn_exp2f(sc[i]);
    if (i & 1) {
      pc[i >> 1] = pack_bf16(e_prev, e);
      sum += e_prev + e;
      asm volatile("" : "+v"(sum), "+v"(pc[i >> 1]));  // here, not wherever the value is first needed
    } else {
      e_prev = e;
    }
    hook(i);  // the caller's share of other work for this MFMA (staging of later tiles)
    __builtin_amdgcn_sched_barrier(0);
  }
  acc = sum;
#pragma unroll
  for (int j = 0; j < kAhead; ++j) {
    if constexpr (NEXT_K) kf[j] = ka[8 + j];
    if constexpr (NEXT_V) vf[j] = va[8 + j];
  }
}

// The general form of one block after the fact: true maximum, base moved to it when it is above the base, P and its
// sum again.  binit: the base the scores in s are relative to.  Returns whether any lane moved its base.
__device__ __forceinline__ bool pipe_redo_block(const f32x16 (&s)[1], float binit, RowState<1> &st, uint32_t (&pc)[1][8],
                                                float &acc) {
  const float bi[1] = {binit};
  float mt[1], alpha[1], off[1], sum[1];
  block_max<1>(s, 1.f, bi, mt);
  const bool raised = raise_max<1>(mt, st, alpha, 0.f);
  const float m_use = (st.m_run[0] == -INFINITY) ? 0.f : st.m_run[0];
  if (raised) {
    rescale<1>(st, alpha);
    st.base[0] = m_use;
#pragma unroll
    for (int j = 0; j < 16; ++j) st.negb[0][j] = -m_use;
  }
  off[0] = binit - m_use;
  block_probs<1, false>(s, 1.f, off, pc, sum);
  acc = sum[0];
  return raised;
}

// One 64-key tile of the pipelined steady state: slot A (S^T of the tile's block 1, P of block 0, O += block 1 of
// the previous tile) and slot B (S^T of block 0 of the next tile, P of block 1, O += block 0).
//   prev / cur / next: the LDS stages of the three tiles (prev == cur for the first tile, whose pq is zero)
//   hook_a(i), hook_b(i): the caller's work beside MFMA i of slot A / slot B
template <bool NEXT, typename HookA, typename HookB>
__device__ __forceinline__ void pipe_tile(const uint8_t *prev, const uint8_t *cur, const uint8_t *next, PipeCarry &cy,
                                          RowState<1> &st, int ln, int lh, HookA &&hook_a, HookB &&hook_b) {
  const int k_lane = ln * kKRow + lh * 16, v_lane = kKTileBytes + ln * kVRow + lh * 16;
  f32x16 s1[1];
  uint32_t p0[1][8], p1[1][8];
  float acc0, acc1;
  // ---- slot A
  const float base_a = st.base[0];
  pipe_slot<true, NEXT, true, 3>(cur + k_lane + 32 * kKRow, prev + v_lane + 64, next + k_lane, cur + v_lane, cy.kf, cy.vf,
                              st.qf[0], st.negb[0], s1[0], cy.s0[0], cy.pq[0], st.o, p0[0], acc0, hook_a);
  // (the rare-path decisions as 64-bit lane masks: one compare, one scalar or, one branch)
  uint64_t raised_a = 0;
  const uint64_t trig_a = __builtin_amdgcn_ballot_w64(acc0 > kTrigger);
  if ((cy.stale0 | trig_a) != 0) raised_a = pipe_redo_block(cy.s0, cy.bs0, st, p0, acc0) ? ~0ull : 0ull;
  raised_a = (uint64_t)(int64_t)(int32_t)__builtin_amdgcn_readfirstlane((uint32_t)raised_a);  // (uniform: keep it scalar)
  st.l_run[0] += acc0;
  // ---- slot B
  const float base_b = st.base[0];
  f32x16 s0n[1];
  pipe_slot<NEXT, NEXT, true, 1>(next + k_lane, cur + v_lane, next + k_lane + 32 * kKRow, cur + v_lane + 64, cy.kf, cy.vf,
                              st.qf[0], st.negb[0], s0n[0], s1[0], p0[0], st.o, p1[0], acc1, hook_b);
  uint64_t raised_b = 0;
  const uint64_t trig_b = __builtin_amdgcn_ballot_w64(acc1 > kTrigger);
  if ((raised_a | trig_b) != 0) raised_b = pipe_redo_block(s1, base_a, st, p1, acc1) ? ~0ull : 0ull;
  raised_b = (uint64_t)(int64_t)(int32_t)__builtin_amdgcn_readfirstlane((uint32_t)raised_b);
  st.l_run[0] += acc1;
  if constexpr (NEXT) cy.s0[0] = s0n[0];
  cy.bs0 = base_b;
  cy.stale0 = raised_b;
#pragma unroll
  for (int j = 0; j < 8; ++j) cy.pq[0][j] = p1[0][j];
}

// NW wavefronts of RB 32-row blocks each: a row tile of 32*NW*RB rows.  STAGES LDS stages per workgroup:
//   4: fp8 cache, one row block per wavefront: the block-pipelined loop (pipe_tile) over the full prefix tiles; one
//      workgroup per CU.  The shape for large row counts on an fp8 cache.
//   3: tile i is computed on while tile i+1 is resident (its first K fragments are fetched early) and tile i+2 is
//      written; one workgroup per CU.  The shape for large row counts on a bf16 cache (whose staging registers leave
//      no room for the pipelined loop's second register set).
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
  const ChunkSel sel = attn_select_chunk(p, id / p.n_row_tiles);
  const int b = sel.b, n_chunks = sel.n_chunks, c = sel.c, k_begin = sel.k_begin, k_end = sel.k_end;
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

  // a wavefront whose rows all lie past R stages tiles but computes nothing (two- and four-stage loops; the
  // three-stage loop computes on every wavefront)
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
      // the chunk K holds at position 2t + lh
      u32x4 v = *(const u32x4 *)(qrow + (KV_FP8 ? k_chunk_at(2 * t + lh) : 2 * t + lh) * 16);
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
  if constexpr (STAGES == 4) {
    // ring of four stages, block-pipelined (see pipe_tile).  Iteration i: the global loads of tile i+2 are in flight;
    // K of tile i (block 1) and of tile i+1 (block 0), V of tile i-1 (block 1) and of tile i (block 0) are read; tile
    // i+2 is written to stage (i+2)%4, which held tile i-2.
    static_assert(STAGES != 4 || RB == 1, "the pipelined loop keeps one row block per wavefront");
    if (n_full > 0) {
      TileRegs<KV_FP8, NT> regs;
      PrefixLoader<KV_FP8, NT> loader;
      loader.init(p, pre, tid);
      auto gload = [&](int it) { loader.load(k_begin + it * kTileN, regs); };
      TileRegs<KV_FP8, NT> regs2;
      // the first tiles are requested together (one round trip to memory, not one per tile)
      gload(0);
      if (n_full > 1) loader.load(k_begin + kTileN, regs2);
      tile_store<KV_FP8, NT>(lds, tid, regs);
      if (n_full > 2) gload(2);  // stays in regs until the loop writes it
      if (n_full > 1) tile_store<KV_FP8, NT>(lds + kStageBytes, tid, regs2);
      __syncthreads();
      PipeCarry cy;
      if (active) {  // S^T of block 0 of tile 0, and the first fragments of slot A of tile 0
        const uint8_t *krow = lds + ln * kKRow + lh * 16;
        const uint8_t *vrow = lds + kKTileBytes + ln * kVRow + lh * 16;
#pragma unroll
        for (int t = 0; t < 8; ++t) k0[t] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(krow + t * 32));
#pragma unroll
        for (int t = 0; t < 8; ++t)
          cy.s0[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0[t], st.qf[0][t], t == 0 ? st.negb[0] : cy.s0[0], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < kAhead; ++t) {
          cy.kf[t] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(krow + 32 * kKRow + t * 32));
          cy.vf[t] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(vrow + 64 + (t & 3) * 32 * kVRow + (t >> 2) * 32));
        }
        cy.bs0 = 0.f;
        cy.stale0 = ~0ull;
#pragma unroll
        for (int j = 0; j < 8; ++j) cy.pq[0][j] = 0u;
      }
      auto stage = [&](int it) { return lds + (it & 3) * kStageBytes; };
      // Staging beside the MFMAs: iteration i requests tile i+3 from global memory during its slot A (block ids from
      // LDS, then the K load, then the V loads) and writes tile i+2, requested an iteration earlier into the other
      // register set, to its stage during slot B; the loads have more than a tile time to arrive.
      int ids[PrefixLoader<KV_FP8, NT>::kNK + PrefixLoader<KV_FP8, NT>::kNV];
      auto no_hook = [](int) {};
      constexpr int kLoads = PrefixLoader<KV_FP8, NT>::kNK + 4 * PrefixLoader<KV_FP8, NT>::kNV;  // per tile and thread
      // one steady-state iteration: the loads of tile it+3 go to `ld`, tile it+2 is written from `stq`
      // (ACT: the wavefront has rows.  A compile-time flag, and one loop per value below: in a loop shared by both
      // kinds of wavefront the compiler hoists the staging conversions the two paths have in common above the branch,
      // and with them the wait for the loads, to the top of the iteration)
      auto steady = [&](auto act, int it, TileRegs<KV_FP8, NT> &ld, const TileRegs<KV_FP8, NT> &stq) __attribute__((always_inline)) {
        const int first = k_begin + (it + 3) * kTileN;
        uint8_t *dst = lds + ((it + 2) & 3) * kStageBytes;
        auto hook_a = [&](int i) __attribute__((always_inline)) {
          if (i == 1) loader.fetch_ids(first, ids);
          if (i == 6) loader.load_k(first, ids, ld);
          if (i == 8) loader.load_v(first, ids, ld);
        };
        auto hook_b = [&](int i) __attribute__((always_inline)) {
          // the loads into stq are older than the kLoads loads into ld just issued; loads return in order
          if (i == 6) {
            __builtin_amdgcn_s_waitcnt((kLoads & 15) | ((kLoads >> 4) << 14) | 0x70 | 0xF00);  // vmcnt(kLoads)
            tile_store_k<KV_FP8, NT>(dst, tid, stq);
          }
          if (i == 9) tile_store_v<KV_FP8, NT, 0>(dst, tid, stq);
          if (i == 12) tile_store_v<KV_FP8, NT, 1>(dst, tid, stq);
        };
        if constexpr (decltype(act)::value) {
          pipe_tile<true>(stage(it > 0 ? it - 1 : 0), stage(it), stage(it + 1), cy, st, ln, lh, hook_a, hook_b);
        } else {  // no rows: only the wavefront's share of the staging
          hook_a(1), hook_a(6), hook_a(8);
          hook_b(6), hook_b(9), hook_b(12);
        }
        __syncthreads();
      };
      int it = 0;
      if (active) {
        for (; it + 4 < n_full; it += 2) {  // steady state, two tiles per trip (the register sets alternate)
          steady(std::true_type{}, it, regs2, regs);
          steady(std::true_type{}, it + 1, regs, regs2);
        }
      } else {
        for (; it + 4 < n_full; it += 2) {
          steady(std::false_type{}, it, regs2, regs);
          steady(std::false_type{}, it + 1, regs, regs2);
        }
        // (no load of this loop is in flight past this point as far as the compiler can tell: it follows the two
        // loops one after the other and would otherwise guard the other loop's registers against these loads with a
        // full wait at the top of its every iteration)
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
      }
      // the last tiles that still have something to write (regs holds tile it+2), then the second to last tile
      for (; it + 1 < n_full; ++it) {
        if (active)
          pipe_tile<true>(stage(it > 0 ? it - 1 : 0), stage(it), stage(it + 1), cy, st, ln, lh, no_hook, no_hook);
        if (it + 2 < n_full) {
          tile_store<KV_FP8, NT>(lds + ((it + 2) & 3) * kStageBytes, tid, regs);
          if (it + 3 < n_full) gload(it + 3);
          __syncthreads();
        }
      }
      if (active) pipe_tile<false>(stage(it > 0 ? it - 1 : 0), stage(it), stage(it), cy, st, ln, lh, no_hook, no_hook);
      if (active) {  // drain: block 1 of the last tile into O
        const uint8_t *vrow = stage(it) + kKTileBytes + ln * kVRow + lh * 16 + 64;
        const u32x4 pw0 = {cy.pq[0][0], cy.pq[0][1], cy.pq[0][2], cy.pq[0][3]};
        const u32x4 pw1 = {cy.pq[0][4], cy.pq[0][5], cy.pq[0][6], cy.pq[0][7]};
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const bf16x8 vu = u < kAhead ? cy.vf[u < kAhead ? u : 0]
                                       : __builtin_bit_cast(bf16x8, *(const u32x4 *)(vrow + (u & 3) * 32 * kVRow + (u >> 2) * 32));
          st.o[u & 3][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vu, __builtin_bit_cast(bf16x8, u < 4 ? pw0 : pw1),
                                                                   st.o[u & 3][0], 0, 0, 0);
        }
      }
      __syncthreads();
    }
  } else if constexpr (STAGES == 3) {
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
    // Loads return in order, so a touch must not be waited for before two more tiles have passed: its value is
    // folded in two iterations later (two variables, the loop unrolled by two so that neither is ever copied),
    // and there is one loop per kind of wavefront (with rows, or staging only): in a shared loop the fragment
    // registers of the computing path and the staging registers of the other overlap, and the compiler then waits
    // for every load in flight before the first fragment read of a tile.
    uint32_t sink = 0;
    if (n_full > 0) {
      TileRegs<KV_FP8, NT> regs;
      PrefixLoader<KV_FP8, NT> loader;
      loader.init(p, pre, tid);
      auto gload = [&](int it) { loader.load(k_begin + it * kTileN, regs); };
      constexpr int kLinesPerRow = kv_row / 128;       // 1 (fp8) or 2 (bf16)
      constexpr int kLines = kTileN * kLinesPerRow;    // lines of the K tile; the V tile has as many
      static_assert(2 * kLines <= NT, "one touch per thread");
      // (unconditional: past the last tile the last one is touched again, and with more threads than lines the
      // lines are touched twice; a load under a branch would have its value copied at the end of the iteration, and
      // the copy waited for)
      const int tline = tid % kLines;
      const uint8_t *const tbase = ((tid / kLines) & 1) ? pre.v_base : pre.k_base;
      auto touch = [&](int it) -> uint32_t {
        const int first = k_begin + min(it, n_full - 1) * kTileN;
        return *(const uint32_t *)(key_row<KV_FP8, true>(p, pre, tbase, first + tline / kLinesPerRow) +
                                   (tline % kLinesPerRow) * 128);
      };
      const uint32_t t1 = touch(1), t2 = touch(2), t3 = touch(3);
      gload(0);
      tile_store<KV_FP8, NT>(lds, tid, regs);
      if (n_full > 1) gload(1);
      uint32_t pfa = t1 ^ t2, pfb = t3;
      __syncthreads();
      // SURE: tiles it+1 and it+2 exist
      auto iter = [&](auto act, auto sure, int it, uint32_t &pf) __attribute__((always_inline)) {
        const uint8_t *cur = lds + (it & 1) * kStageBytes;
        uint8_t *other = lds + ((it + 1) & 1) * kStageBytes;
        auto tail = [&] {
          if (decltype(sure)::value || it + 1 < n_full) {
            tile_store<KV_FP8, NT>(other, tid, regs);
            if (decltype(sure)::value || it + 2 < n_full) gload(it + 2);
          }
          sink ^= pf;  // requested two iterations ago
          __builtin_amdgcn_sched_barrier(0);  // (the old value is dead before the new load is issued)
          pf = touch(it + 4);
        };
        if constexpr (decltype(act)::value)
          compute_tile<RB, MASK_NONE, false, false>(cur, nullptr, k0, st, ln, lh, 0, 0, 1.f, 0.f, 1.f, tail);
        else
          tail();
        __syncthreads();
      };
      auto tiles = [&](auto act) __attribute__((always_inline)) {
        int it = 0;
        for (; it + 3 < n_full; it += 2) {  // steady state: no load is conditional
          iter(act, std::true_type{}, it, pfa);
          iter(act, std::true_type{}, it + 1, pfb);
        }
        for (; it < n_full; ++it) iter(act, std::false_type{}, it, (it & 1) ? pfb : pfa);
      };
      if (active) {
        tiles(std::true_type{});
      } else {
        tiles(std::false_type{});
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): see the four-stage loop
      }
      sink ^= pfa ^ pfb;
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
        tile_load<BR_FP8, false, false, NT, KV_FP8>(p, pool, tid, regs);
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
    tile_load<BR_FP8, false, false, NT, KV_FP8>(p, src, tid, bregs);
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

// STAGES: LDS stages with a bf16 cache; an fp8 cache (half the staging registers) with three or more stages runs
// the block-pipelined loop on four stages instead.
template <int NW, int RB, int STAGES>
hipError_t launch_shape(const AttnParams &p, bool kv_fp8, bool br_fp8, hipStream_t stream) {
  constexpr int kFp8Stages = (STAGES >= 3 && RB == 1) ? 4 : STAGES;
  if (p.C > 0 && p.pool_seg) {
    if (kv_fp8 && br_fp8) return launch_variant<true, true, NW, RB, kFp8Stages, 2>(p, stream);
    if (kv_fp8 && !br_fp8) return launch_variant<true, false, NW, RB, kFp8Stages, 2>(p, stream);
    if (!kv_fp8 && !br_fp8) return launch_variant<false, false, NW, RB, STAGES, 2>(p, stream);
    return hipErrorInvalidValue;
  }
  if (p.C > 0) {
    if (kv_fp8 && br_fp8) return launch_variant<true, true, NW, RB, kFp8Stages, 1>(p, stream);
    if (kv_fp8 && !br_fp8) return launch_variant<true, false, NW, RB, kFp8Stages, 1>(p, stream);
    if (!kv_fp8 && !br_fp8) return launch_variant<false, false, NW, RB, STAGES, 1>(p, stream);
    return hipErrorInvalidValue;
  }
  if (kv_fp8 && br_fp8) return launch_variant<true, true, NW, RB, kFp8Stages, 0>(p, stream);
  if (kv_fp8 && !br_fp8) return launch_variant<true, false, NW, RB, kFp8Stages, 0>(p, stream);
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
