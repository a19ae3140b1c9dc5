// Device helpers shared by the verify-attention MFMA kernels (gfx950).
#pragma once

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

// A running maximum is only raised when the tile maximum exceeds it by more than this many log2 units; until
// then probabilities are allowed to reach 2^kRaise, which fp32 sums and bf16 operands hold without loss.  Raising
// rarely keeps the accumulator rescale (64 multiplies per lane and row block) off the common path.
constexpr float kRaise = 6.0f;


// Per-wavefront state of RB blocks of 32 query rows.
template <int RB>
struct RowState {
  bf16x8 qf[RB][8];  // Q^T operand, already multiplied by the prefix score scale (log2 units): row ln of block rb,
                     // d = 16t + 8*lh .. +8
  f32x16 o[4][RB];   // O^T accumulators: d block db, row block rb
  f32x16 negb[RB];   // every element = -base: the accumulator a full prefix tile's S^T starts from, so that the
                     // MFMAs deliver s - base directly
  float base[RB];    // == m_run once a maximum exists, 0 before
  float m_run[RB], l_run[RB];
  int row_tok[RB], row_bstart[RB];
  // tree form only: the segments the row's branch sees, and (lane k) the segment of key k of the current pool tile
  uint64_t row_mask[RB];
  int tile_seg;
};

enum MaskMode { MASK_NONE = 0, MASK_TAIL = 1, MASK_BRANCH = 2, MASK_TREE = 3 };

// sched_group_barrier masks
constexpr int kSgMfma = 0x008, kSgValu = 0x002, kSgSalu = 0x004, kSgVmemRead = 0x020, kSgDsRead = 0x100;

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
  } else if constexpr (MASK == MASK_TREE) {
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int ka = kb * 32 + (j >> 2) * 8 + (j & 3);  // this register's key in the lower lane half; upper: + 4
      const int sa = __builtin_amdgcn_readlane(st.tile_seg, ka), sb = __builtin_amdgcn_readlane(st.tile_seg, ka + 4);
      const int seg = lh ? sb : sa;
      const bool past = first + ka + lh * 4 >= limit;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        if (past || !((st.row_mask[rb] >> seg) & 1)) s[rb][j] = -INFINITY;
    }
  }
}

// Absolute maximum (log2 units) of one 32-key block per row.  The scores arrive as x with absolute value
// x*crel + binit (binit: what the accumulators were started from, per lane).
template <int RB>
__device__ __forceinline__ void block_max(const f32x16 (&s)[RB], float crel, const float (&binit)[RB],
                                          float (&mt)[RB]) {
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float ma = fmaxf(fmaxf(s[rb][0], s[rb][1]), s[rb][2]);
    float mb = fmaxf(fmaxf(s[rb][8], s[rb][9]), s[rb][10]);
    ma = fmaxf(fmaxf(ma, s[rb][3]), s[rb][4]);
    mb = fmaxf(fmaxf(mb, s[rb][11]), s[rb][12]);
    ma = fmaxf(fmaxf(ma, s[rb][5]), s[rb][6]);
    mb = fmaxf(fmaxf(mb, s[rb][13]), s[rb][14]);
    const float m0 = fmaxf(fmaxf(ma, s[rb][7]), fmaxf(mb, s[rb][15]));
    mt[rb] = __builtin_fmaf(xhalf_max(m0), crel, binit[rb]);
  }
}

// Fold the block maxima into the running maxima.  A lane raises its maximum only when the block exceeds it by more
// than `threshold`; alpha is the factor its old accumulators must then be multiplied by (1 for lanes that keep their
// maximum).  Returns whether any lane of the wavefront raised (wavefront-uniform).
template <int RB>
__device__ __forceinline__ bool raise_max(const float (&mt)[RB], RowState<RB> &st, float (&alpha)[RB],
                                          float threshold = kRaise) {
  bool raise = false;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const bool up = mt[rb] > st.m_run[rb] + threshold;   // false for mt = -inf; true for the first finite block
    const float m_new = up ? mt[rb] : st.m_run[rb];
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

// p = 2^(x*crel + off) for one 32-key block, rounded to bf16 pairs; also the fp32 row sums.  off = binit + voff - m
// per lane.  FAST: crel == 1 and off == 0 for every lane (accumulators started from -m), so p = 2^x.
template <int RB, bool FAST>
__device__ __forceinline__ void block_probs(const f32x16 (&s)[RB], float crel, const float (&off)[RB],
                                            uint32_t (&pb)[RB][8], float (&sum)[RB]) {
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < 16; j += 2) {
      const float p0 = __builtin_amdgcn_exp2f(FAST ? s[rb][j] : __builtin_fmaf(s[rb][j], crel, off[rb]));
      const float p1 = __builtin_amdgcn_exp2f(FAST ? s[rb][j + 1] : __builtin_fmaf(s[rb][j + 1], crel, off[rb]));
      pb[rb][j >> 1] = pack_bf16(p0, p1);
      // (a v_dot2c_f32_bf16 on the packed pair would sum the rounded values in one instruction, but on gfx950 it
      // stalls against the MFMAs in flight: measured slower than the two adds)
      acc += p0 + p1;
    }
    sum[rb] = acc;
  }
}


// Which request and which of its chunks workgroup-unit `unit` (counted over the chunks of all requests, request by
// request) reduces, and that chunk's key range.  Chunks are numbered from the end: the last chunk of a request (it also
// carries the branch-private tiles and so runs longest) comes first in dispatch order.
struct ChunkSel {
  int b, P, n_chunks, c, k_begin, k_end;
};
__device__ __forceinline__ ChunkSel attn_select_chunk(const AttnParams &p, int unit) {
  ChunkSel s;
  s.b = 0, s.P = 0, s.n_chunks = 1;
  int c = unit;
  if (p.n_inline) {
    // few requests: everything comes from the kernel arguments (indexed with constants only, so that it stays in
    // scalar registers), no load and no division
    int q = 0, r = 0;
    uint32_t inv = 0;
    bool found = false;
#pragma unroll
    for (int i = 0; i < kMaxInlineLens; ++i) {
      if (!found && i < p.B) {
        if (c < p.req[i].n || i == p.B - 1) {
          s.b = i, s.P = p.req[i].P, s.n_chunks = p.req[i].n, q = p.req[i].q, r = p.req[i].r, inv = p.req[i].inv;
          found = true;
        } else {
          c -= p.req[i].n;
        }
      }
    }
    c = s.n_chunks - 1 - c;
    // attn_chunk_range with floor(c * (q*n + r) / n) = c*q + floor(c*r / n) and the quotient by multiply-shift
    const int T = (s.P + 63) >> 6;
    const int t0 = min(T, c * q + (int)__umulhi((uint32_t)(c * r), inv));
    const int t1 = c == s.n_chunks - 1 ? T : min(T, (c + 1) * q + (int)__umulhi((uint32_t)((c + 1) * r), inv));
    s.k_begin = t0 * 64;
    s.k_end = min(s.P, t1 * 64);
  } else {
    int b = 0;
    for (; b < p.B - 1; ++b) {
      const int nc = attn_num_chunks(p.prefix_lens[b], p.chunk_len);
      if (c < nc) break;
      c -= nc;
    }
    s.b = b;
    s.P = p.prefix_lens[b];
    s.n_chunks = attn_num_chunks(s.P, p.chunk_len);
    c = s.n_chunks - 1 - c;
    attn_chunk_range(s.P, p.chunk_len, p.last_short, c, &s.k_begin, &s.k_end);
  }
  s.c = c;
  return s;
}

}  // namespace
}  // namespace la
