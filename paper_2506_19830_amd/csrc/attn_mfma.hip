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
// Per 64-key tile and wave (RB blocks of 32 rows each):
//   S^T = K Q^T      v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q (registers)
//   online softmax   each lane owns one query row (column of S^T): the row max is an
//                    in-lane reduction plus one exchange with lane^32
//   O^T += V^T P^T   A = V^T from LDS (stored transposed, keys permuted inside groups
//                    of 16 so that the accumulator registers of S^T are already the
//                    B operand), B = P^T (registers, bf16)
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
constexpr int kThreads = 256;                // 4 waves
constexpr int kKRow = kD * 2 + 16;           // bytes per key row of the K tile in LDS (padded)
constexpr int kVRow = kTileN * 2 + 16;       // bytes per d row of the V^T tile in LDS (padded)
constexpr int kKTileBytes = kTileN * kKRow;  // 17408
constexpr int kVTileBytes = kD * kVRow;      // 18432
constexpr int kStageBytes = kKTileBytes + kVTileBytes;
constexpr int kLdsBytes = 2 * kStageBytes;   // double buffered: 71680

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}

// two fp8-e4m3 of a 32-bit word (low or high half) -> two floats
template <bool HI>
__device__ __forceinline__ f32x2 fp8x2_to_f32(uint32_t w) {
  return __builtin_amdgcn_cvt_pk_f32_fp8(w, HI);
}

// position of key quad kq (keys 4kq..4kq+3 of the tile) inside a V^T row: inside every group of 16 keys
// key 8a+4h+c sits at 8h+4a+c, which is the order the S^T accumulator registers come in
__device__ __forceinline__ int vt_pos(int kq) { return 16 * (kq >> 2) + 8 * (kq & 1) + 4 * ((kq >> 1) & 1); }

// Where the keys of one tile come from.
struct TileSrc {
  const uint8_t *k_base, *v_base;  // prefix: cache base; branch: row of token 0 of this request and kv head
  const int32_t *table;            // prefix: block table row of the request or null (identity)
  int ident_base;                  // prefix, identity mapping: first physical block of the request
  int first;                       // first key of the tile (prefix: token index; branch: token t = g*L+j)
  int limit;                       // keys >= limit are zero filled
  bool is_prefix;
};

// Staging registers of one K tile and one V tile (per thread): 16 B pieces of K, 4 B pieces of V.
struct TileRegs {
  u32x4 k[4];
  uint32_t v[16];
};

template <bool FP8>
__device__ __forceinline__ const uint8_t *key_row(const AttnParams &p, const TileSrc &s, const uint8_t *base,
                                                  int kvh, int tok) {
  constexpr int esz = FP8 ? 1 : 2;
  if (s.is_prefix) {
    const int lb = tok / p.block_size;
    const int blk = s.table ? s.table[lb] : s.ident_base + lb;
    return base + (((size_t)blk * p.Hkv + kvh) * p.block_size + (tok % p.block_size)) * (size_t)(kD * esz);
  }
  return base + (size_t)tok * p.Hkv * (kD * esz);
}

template <bool FP8>
__device__ __forceinline__ void tile_load(const AttnParams &p, const TileSrc &s, int kvh, int tid, TileRegs &r) {
  if constexpr (!FP8) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {  // K: 16 B = 8 d of key (tid/16 + 16e)
      const int tok = s.first + (tid >> 4) + 16 * e;
      u32x4 val = {0, 0, 0, 0};
      if (tok < s.limit) val = *(const u32x4 *)(key_row<FP8>(p, s, s.k_base, kvh, tok) + (tid & 15) * 16);
      r.k[e] = val;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {  // V: 4 B = d pair (tid%64) of the 4 keys of quad (tid/64 + 4e)
      const int kq = (tid >> 6) + 4 * e;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int tok = s.first + 4 * kq + c;
        uint32_t val = 0;
        if (tok < s.limit) val = *(const uint32_t *)(key_row<FP8>(p, s, s.v_base, kvh, tok) + (tid & 63) * 4);
        r.v[4 * e + c] = val;
      }
    }
  } else {
#pragma unroll
    for (int e = 0; e < 2; ++e) {  // K: 16 B = 16 d of key (tid/8 + 32e)
      const int tok = s.first + (tid >> 3) + 32 * e;
      u32x4 val = {0, 0, 0, 0};
      if (tok < s.limit) val = *(const u32x4 *)(key_row<FP8>(p, s, s.k_base, kvh, tok) + (tid & 7) * 16);
      r.k[e] = val;
    }
#pragma unroll
    for (int e = 0; e < 2; ++e) {  // V: 4 B = d quad (tid%32) of the 4 keys of quad (tid/32 + 8e)
      const int kq = (tid >> 5) + 8 * e;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int tok = s.first + 4 * kq + c;
        uint32_t val = 0;
        if (tok < s.limit) val = *(const uint32_t *)(key_row<FP8>(p, s, s.v_base, kvh, tok) + (tid & 31) * 4);
        r.v[4 * e + c] = val;
      }
    }
  }
}

template <bool FP8>
__device__ __forceinline__ void tile_store(uint8_t *stage, int tid, const TileRegs &r) {
  uint8_t *kt = stage;
  uint8_t *vt = stage + kKTileBytes;
  if constexpr (!FP8) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int key = (tid >> 4) + 16 * e;
      *(u32x4 *)(kt + key * kKRow + (tid & 15) * 16) = r.k[e];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int kq = (tid >> 6) + 4 * e;
      const int d0 = 2 * (tid & 63);
      const uint32_t a = r.v[4 * e + 0], b = r.v[4 * e + 1], c = r.v[4 * e + 2], d = r.v[4 * e + 3];
      // low halves hold d0 of keys (a,b,c,d), high halves d0+1
      u32x2 lo = {__builtin_amdgcn_perm(b, a, 0x05040100u), __builtin_amdgcn_perm(d, c, 0x05040100u)};
      u32x2 hi = {__builtin_amdgcn_perm(b, a, 0x07060302u), __builtin_amdgcn_perm(d, c, 0x07060302u)};
      *(u32x2 *)(vt + d0 * kVRow + vt_pos(kq) * 2) = lo;
      *(u32x2 *)(vt + (d0 + 1) * kVRow + vt_pos(kq) * 2) = hi;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int key = (tid >> 3) + 32 * e;
      uint32_t out[8];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const f32x2 lo = fp8x2_to_f32<false>(r.k[e][w]);
        const f32x2 hi = fp8x2_to_f32<true>(r.k[e][w]);
        out[2 * w] = pack_bf16(lo.x, lo.y);
        out[2 * w + 1] = pack_bf16(hi.x, hi.y);
      }
      uint8_t *dst = kt + key * kKRow + (tid & 7) * 32;
      *(u32x4 *)(dst) = u32x4{out[0], out[1], out[2], out[3]};
      *(u32x4 *)(dst + 16) = u32x4{out[4], out[5], out[6], out[7]};
    }
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int kq = (tid >> 5) + 8 * e;
      const int d0 = 4 * (tid & 31);
      f32x2 lo[4], hi[4];  // of key c: (d0, d0+1) and (d0+2, d0+3)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        lo[c] = fp8x2_to_f32<false>(r.v[4 * e + c]);
        hi[c] = fp8x2_to_f32<true>(r.v[4 * e + c]);
      }
      uint8_t *dst = vt + d0 * kVRow + vt_pos(kq) * 2;
      *(u32x2 *)(dst) = u32x2{pack_bf16(lo[0].x, lo[1].x), pack_bf16(lo[2].x, lo[3].x)};
      *(u32x2 *)(dst + kVRow) = u32x2{pack_bf16(lo[0].y, lo[1].y), pack_bf16(lo[2].y, lo[3].y)};
      *(u32x2 *)(dst + 2 * kVRow) = u32x2{pack_bf16(hi[0].x, hi[1].x), pack_bf16(hi[2].x, hi[3].x)};
      *(u32x2 *)(dst + 3 * kVRow) = u32x2{pack_bf16(hi[0].y, hi[1].y), pack_bf16(hi[2].y, hi[3].y)};
    }
  }
}

template <bool KV_FP8, bool BR_FP8, int RB>
__global__ __launch_bounds__(kThreads, RB == 1 ? 2 : 1) void attn_mfma_kernel(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  constexpr int kTileM = 128 * RB;
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
  const int n_prefix_tiles = k_end > k_begin ? (k_end - k_begin + kTileN - 1) / kTileN : 0;

  const int r0 = row_tile * kTileM;
  const int r1 = min(p.R, r0 + kTileM);
  const int gl = p.gamma * p.L;
  // branch-private keys needed by this row tile: tokens t = g*L + j in [tk0, t_hi]
  const int t_lo = r0 / p.G, t_hi = (r1 - 1) / p.G;
  const int tk0 = (t_lo / p.L) * p.L;
  const int n_priv_tiles = (c == n_chunks - 1) ? (t_hi - tk0 + 1 + kTileN - 1) / kTileN : 0;
  const int n_tiles = n_prefix_tiles + n_priv_tiles;

  constexpr int br_esz = BR_FP8 ? 1 : 2;
  const size_t br_off = ((size_t)b * gl * p.Hkv + kvh) * (kD * br_esz);

  auto tile_src = [&](int it) {
    TileSrc s;
    if (it < n_prefix_tiles) {
      s.is_prefix = true;
      s.first = k_begin + it * kTileN;
      s.limit = k_end;
      s.k_base = (const uint8_t *)p.k_cache;
      s.v_base = (const uint8_t *)p.v_cache;
      s.table = p.block_tables ? p.block_tables + (size_t)b * p.max_blocks : nullptr;
      s.ident_base = b * p.max_blocks;
    } else {
      s.is_prefix = false;
      s.first = tk0 + (it - n_prefix_tiles) * kTileN;
      s.limit = t_hi + 1;
      s.k_base = (const uint8_t *)p.k_branch + br_off;
      s.v_base = (const uint8_t *)p.v_branch + br_off;
      s.table = nullptr;
      s.ident_base = 0;
    }
    return s;
  };
  auto load_tile = [&](int it, TileRegs &regs) {
    const TileSrc s = tile_src(it);
    if (s.is_prefix)
      tile_load<KV_FP8>(p, s, kvh, tid, regs);
    else
      tile_load<BR_FP8>(p, s, kvh, tid, regs);
  };
  auto store_tile = [&](int it, const TileRegs &regs) {
    uint8_t *stage = lds + (it & 1) * kStageBytes;
    if (it < n_prefix_tiles)
      tile_store<KV_FP8>(stage, tid, regs);
    else
      tile_store<BR_FP8>(stage, tid, regs);
  };

  // ---- per-lane query rows ---------------------------------------------------------------
  int row[RB], row_tok[RB], row_bstart[RB];
  bf16x8 qf[RB][8];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int r = r0 + (wave * RB + rb) * 32 + ln;
    row[rb] = r;
    const int rr = min(r, p.R - 1);
    row_tok[rb] = rr / p.G;
    row_bstart[rb] = (row_tok[rb] / p.L) * p.L;
    const uint8_t *qrow =
        (const uint8_t *)p.q + (((size_t)b * gl + row_tok[rb]) * p.Hq + kvh * p.G + (rr % p.G)) * (size_t)(kD * 2);
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      u32x4 v = {0, 0, 0, 0};
      if (r < p.R) v = *(const u32x4 *)(qrow + (16 * t + 8 * lh) * 2);
      qf[rb][t] = __builtin_bit_cast(bf16x8, v);
    }
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

  f32x16 o[4][RB];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int j = 0; j < 16; ++j) o[db][rb][j] = 0.f;
  float m_run[RB], l_run[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) m_run[rb] = -INFINITY, l_run[rb] = 0.f;

  // ---- pipeline prologue -------------------------------------------------------------------
  TileRegs regs;
  if (n_tiles > 0) {
    load_tile(0, regs);
    store_tile(0, regs);
  }
  __syncthreads();

  for (int it = 0; it < n_tiles; ++it) {
    const bool has_next = it + 1 < n_tiles;
    if (has_next) load_tile(it + 1, regs);

    const uint8_t *kt = lds + (it & 1) * kStageBytes;
    const uint8_t *vt = kt + kKTileBytes;
    const bool is_prefix = it < n_prefix_tiles;
    const int first = is_prefix ? k_begin + it * kTileN : tk0 + (it - n_prefix_tiles) * kTileN;

    // ---- S^T = K Q^T -------------------------------------------------------------------
    f32x16 s[2][RB];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int j = 0; j < 16; ++j) s[kb][rb][j] = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      bf16x8 kf[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
        kf[kb] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(kt + (kb * 32 + ln) * kKRow + (16 * t + 8 * lh) * 2));
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          s[kb][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb], qf[rb][t], s[kb][rb], 0, 0, 0);
    }

    // ---- mask --------------------------------------------------------------------------
    // register j of block kb holds key  kb*32 + (j/4)*8 + lh*4 + j%4  of the tile
    if (is_prefix) {
      if (first + kTileN > k_end) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            const int key = first + kb * 32 + (j >> 2) * 8 + lh * 4 + (j & 3);
            if (key >= k_end) {
#pragma unroll
              for (int rb = 0; rb < RB; ++rb) s[kb][rb][j] = -INFINITY;
            }
          }
      }
    } else {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int tk = first + kb * 32 + (j >> 2) * 8 + lh * 4 + (j & 3);
#pragma unroll
          for (int rb = 0; rb < RB; ++rb)
            if (tk > row_tok[rb] || tk < row_bstart[rb]) s[kb][rb][j] = -INFINITY;
        }
    }

    // ---- online softmax ------------------------------------------------------------------
    const float cseg = is_prefix ? c_prefix : c_branch;
    const float voff = is_prefix ? 0.f : voff_branch;
    const float lmul = is_prefix ? 1.f : lmul_branch;
    uint32_t pb[2][RB][8];  // P^T as bf16 pairs: [kb][rb][j/2]
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      float mt = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int j = 0; j < 16; ++j) mt = fmaxf(mt, s[kb][rb][j]);
      mt = fmaxf(mt, __shfl_xor(mt, 32));
      const float m_new = fmaxf(m_run[rb], mt * cseg);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run[rb] - m_use);
      m_run[rb] = m_new;
      const float off = voff - m_use;
      float sum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int j = 0; j < 16; j += 2) {
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][rb][j], cseg, off));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][rb][j + 1], cseg, off));
          sum += p0 + p1;
          pb[kb][rb][j >> 1] = pack_bf16(p0, p1);
        }
      l_run[rb] = l_run[rb] * alpha + sum * lmul;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[db][rb][j] *= alpha;
    }

    // ---- O^T += V^T P^T ------------------------------------------------------------------
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        bf16x8 pf[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          u32x4 v = {pb[kb][rb][4 * t2], pb[kb][rb][4 * t2 + 1], pb[kb][rb][4 * t2 + 2], pb[kb][rb][4 * t2 + 3]};
          pf[rb] = __builtin_bit_cast(bf16x8, v);
        }
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const bf16x8 vf = __builtin_bit_cast(
              bf16x8, *(const u32x4 *)(vt + (db * 32 + ln) * kVRow + (kb * 32 + t2 * 16 + lh * 8) * 2));
#pragma unroll
          for (int rb = 0; rb < RB; ++rb)
            o[db][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[rb], o[db][rb], 0, 0, 0);
        }
      }

    if (has_next) store_tile(it + 1, regs);
    __syncthreads();
  }

  // ---- write the partial -----------------------------------------------------------------
  const size_t slot = (size_t)b * p.s_max + c;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const float l_tot = l_run[rb] + __shfl_xor(l_run[rb], 32);
    if (row[rb] < p.R) {
      const size_t out_row = slot * p.n_rows + (size_t)row_tok[rb] * p.Hq + kvh * p.G + (row[rb] % p.G);
      float *po = p.part_o + out_row * kD;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          f32x4 v = {o[db][rb][4 * q4] * v_out, o[db][rb][4 * q4 + 1] * v_out, o[db][rb][4 * q4 + 2] * v_out,
                     o[db][rb][4 * q4 + 3] * v_out};
          *(f32x4 *)(po + db * 32 + q4 * 8 + lh * 4) = v;
        }
      if (lh == 0) {
        f32x2 ml = {m_run[rb], l_tot};
        *(f32x2 *)(p.part_ml + out_row * 2) = ml;
      }
    }
  }
}

template <bool KV_FP8, bool BR_FP8, int RB>
hipError_t launch_variant(const AttnParams &p, hipStream_t stream) {
  const int grid = p.Hkv * p.n_row_tiles * p.total_units;
  auto kern = attn_mfma_kernel<KV_FP8, BR_FP8, RB>;
  hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), kLdsBytes, stream, p);
  return hipGetLastError();
}

}  // namespace

int attn_mfma_tile_m(int R) {
  (void)R;
  return 256;
}

hipError_t launch_attn_mfma(const AttnParams &p, bool kv_fp8, bool br_fp8, hipStream_t stream) {
  ProfileScope scope(SLOT_ATTN_MFMA, stream);
  if (kv_fp8 && br_fp8) return launch_variant<true, true, 2>(p, stream);
  if (kv_fp8 && !br_fp8) return launch_variant<true, false, 2>(p, stream);
  if (!kv_fp8 && !br_fp8) return launch_variant<false, false, 2>(p, stream);
  return hipErrorInvalidValue;
}

}  // namespace la
