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

}  // namespace
}  // namespace la
