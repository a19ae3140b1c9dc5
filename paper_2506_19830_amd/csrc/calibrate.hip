// Calibration kernels for the benchmark (not part of the verification path): what this very chip reaches on a
// pure bf16 MFMA loop and on a pure streaming read, so that a roofline fraction can be quoted against the
// achievable rate next to the published peak; and an instruction-mix probe (la_calibrate_issue) that measures how
// fast a wavefront, and two wavefronts sharing a SIMD, issue the instruction kinds the attention kernels are made of.
#include "la_internal.hpp"
#include "la_verify_bench.h"

namespace la {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kCalibChains = 4;  // independent accumulators per wavefront

// 8 wavefronts per workgroup, each running kCalibChains independent v_mfma_f32_32x32x16_bf16 chains.
__global__ __launch_bounds__(512) void calib_mfma_kernel(float *sink, int iters) {
  const float seed = 1.0f + (float)(threadIdx.x & 7) * 0.125f;
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(seed * 0.01f);
    b[i] = (__bf16)(0.02f - seed * 0.001f);
  }
  f32x16 acc[kCalibChains];
#pragma unroll
  for (int c = 0; c < kCalibChains; ++c)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[c][j] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int c = 0; c < kCalibChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kCalibChains; ++c)
#pragma unroll
    for (int j = 0; j < 16; ++j) s += acc[c][j];
  sink[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

// The same loop on operands that look like data: eight operand pairs per lane, every element a different
// pseudo-random bf16 in (-2, 2), used in rotation, so that the operand paths and multipliers of the matrix pipeline
// toggle as they do on a real K/V stream.  On a chip whose clock is power-managed this is the rate to compare a
// kernel's MFMA throughput with; the loop above (nearly constant operands) shows the top clock.
__global__ __launch_bounds__(512) void calib_mfma_data_kernel(float *sink, int iters) {
  bf16x8 a[8], b[8];
  uint32_t h = (blockIdx.x * 512u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int k = 0; k < 8; ++k)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      h = h * 1664525u + 1013904223u;  // a linear congruential step per element; the high bits are used
      a[k][i] = (__bf16)((float)((int)(h >> 16) - 32768) * (1.0f / 16384.0f));
      h = h * 1664525u + 1013904223u;
      b[k][i] = (__bf16)((float)((int)(h >> 16) - 32768) * (1.0f / 16384.0f));
    }
  f32x16 acc[kCalibChains];
#pragma unroll
  for (int c = 0; c < kCalibChains; ++c)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[c][j] = 0.f;
  for (int it = 0; it < iters; it += 2) {  // two rounds per trip: consecutive MFMAs never share an operand
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
      for (int c = 0; c < kCalibChains; ++c) {
        constexpr int kB[8] = {3, 4, 5, 6, 7, 0, 1, 2};
        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c + 4 * r], b[kB[c + 4 * r]], acc[c], 0, 0, 0);
      }
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kCalibChains; ++c)
#pragma unroll
    for (int j = 0; j < 16; ++j) s += acc[c][j];
  sink[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

// Grid-stride streaming read, eight 16-byte loads in flight per thread; the data only feeds an xor.
__global__ __launch_bounds__(256) void calib_read_kernel(const u32x4 *src, size_t n16, uint32_t *sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  u32x4 x = {0, 0, 0, 0};
  for (; i + 7 * stride < n16; i += 8 * stride) {
    u32x4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(src + i + j * stride);
#pragma unroll
    for (int j = 0; j < 8; ++j) x ^= v[j];
  }
  for (; i < n16; i += stride) x ^= src[i];
  const uint32_t w = x[0] ^ x[1] ^ x[2] ^ x[3];
  if (w == 0x9e3779b9u) sink[0] = w;  // practically never: keeps the loads alive without a store on the real path
}

// ---- instruction-mix probe ------------------------------------------------------------------------------------------
// 4 or 8 wavefronts per workgroup (one or two per SIMD), one workgroup per CU.  Every wavefront runs `iters` rounds of a
// body of 16 slots; what a slot holds depends on the mix.  With 8 wavefronts the second wavefront of each SIMD
// (wavefronts 4..7) may run another mix than the first.  No memory access besides one store per lane at the end.
enum IssueMix {
  MIX_ADD = 0,        // slot = v_add_f32
  MIX_EXP,            // slot = v_exp_f32
  MIX_CVT,            // slot = v_cvt_pk_bf16_f32
  MIX_MFMA,           // slot = MFMA, four accumulators in turn, one pair of operand registers
  MIX_MFMA_OPERANDS,  // slot = MFMA, four accumulators in turn, eight different operand register pairs
  MIX_MFMA_ADD4,      // slot = MFMA + 4 v_add_f32
  MIX_MFMA_ADD8,      // slot = MFMA + 8 v_add_f32
  MIX_MFMA_SOFTMAX,   // slot = MFMA + v_exp_f32 + (every other slot) v_cvt_pk_bf16_f32 + 2 v_add_f32
  MIX_COUNT
};

#define LA_REP8(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7)

template <int MIX>
__device__ __forceinline__ void issue_body(float (&x)[8], f32x16 (&acc)[4], const bf16x8 (&av)[8], const bf16x8 (&bv)[8]) {
  if constexpr (MIX == MIX_ADD) {
#define X(i) asm volatile("v_add_f32 %0, %0, %1" : "+v"(x[i]) : "v"(x[(i + 1) & 7]));
    LA_REP8(X) LA_REP8(X)
#undef X
  } else if constexpr (MIX == MIX_EXP) {
#define X(i) asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
    LA_REP8(X) LA_REP8(X)
#undef X
  } else if constexpr (MIX == MIX_CVT) {
#define X(i) asm volatile("v_cvt_pk_bf16_f32 %0, %0, %1" : "+v"(x[i]) : "v"(x[(i + 1) & 7]));
    LA_REP8(X) LA_REP8(X)
#undef X
  } else {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int r = MIX == MIX_MFMA ? 0 : (i & 7);
      acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[r], bv[(r + 3) & 7], acc[i & 3], 0, 0, 0);
      asm volatile("" : "+v"(acc[i & 3]));
      if constexpr (MIX == MIX_MFMA_ADD4 || MIX == MIX_MFMA_ADD8) {
#define X(j) \
  if (j < (MIX == MIX_MFMA_ADD4 ? 4 : 8)) asm volatile("v_add_f32 %0, %0, %1" : "+v"(x[j]) : "v"(x[(j + 1) & 7]));
        LA_REP8(X)
#undef X
      }
      if constexpr (MIX == MIX_MFMA_SOFTMAX) {
        asm volatile("v_exp_f32 %0, %0" : "+v"(x[i & 1]));
        if (i & 1) {
          asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(x[2]) : "v"(x[0]), "v"(x[1]));
          asm volatile("v_add_f32 %0, %1, %2" : "=v"(x[3]) : "v"(x[0]), "v"(x[1]));
          asm volatile("v_add_f32 %0, %0, %1" : "+v"(x[4]) : "v"(x[3]));
        }
      }
    }
  }
}

template <int MIX_A, int MIX_B>
__global__ __launch_bounds__(512) void calib_issue_kernel(float *sink, int iters) {
  float x[8];
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = -1.0f - (float)(threadIdx.x & 15) * 1e-3f - (float)i;
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[c][j] = 0.f;
  bf16x8 av[8], bv[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      av[r][i] = (__bf16)(0.01f + 0.001f * (float)r);
      bv[r][i] = (__bf16)(0.02f - 0.001f * (float)r);
    }
    asm volatile("" : "+v"(av[r]), "+v"(bv[r]));
  }
  if ((threadIdx.x >> 6) < 4) {
    for (int it = 0; it < iters; ++it) issue_body<MIX_A>(x, acc, av, bv);
  } else {
    for (int it = 0; it < iters; ++it) issue_body<MIX_B>(x, acc, av, bv);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += x[i];
#pragma unroll
  for (int c = 0; c < 4; ++c) s += acc[c][0] + acc[c][7];
  sink[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

template <int A, int B>
void launch_issue(int workgroups, int waves, int iters, float *sink, hipStream_t stream) {
  hipLaunchKernelGGL((calib_issue_kernel<A, B>), dim3(workgroups), dim3(64 * waves), 0, stream, sink, iters);
}

}  // namespace
}  // namespace la

using namespace la;

extern "C" {

la_status la_calibrate_mfma(int32_t workgroups, int32_t iters, float *sink, double *flops, void *hip_stream) {
  if (workgroups < 1 || workgroups > (1 << 20) || iters < 1 || !sink || !flops) return LA_ERR_INVALID_ARG;
  {
    ProfileScope scope(SLOT_CALIB_MFMA, (hipStream_t)hip_stream);
    hipLaunchKernelGGL(calib_mfma_kernel, dim3(workgroups), dim3(512), 0, (hipStream_t)hip_stream, sink, iters);
  }
  *flops = (double)workgroups * 8 * kCalibChains * (double)iters * 2.0 * 32 * 32 * 16;
  return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

la_status la_calibrate_mfma_data(int32_t workgroups, int32_t iters, float *sink, double *flops, void *hip_stream) {
  if (workgroups < 1 || workgroups > (1 << 20) || iters < 2 || (iters & 1) || !sink || !flops) return LA_ERR_INVALID_ARG;
  {
    ProfileScope scope(SLOT_CALIB_MFMA, (hipStream_t)hip_stream);
    hipLaunchKernelGGL(calib_mfma_data_kernel, dim3(workgroups), dim3(512), 0, (hipStream_t)hip_stream, sink, iters);
  }
  *flops = (double)workgroups * 8 * kCalibChains * (double)iters * 2.0 * 32 * 32 * 16;
  return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

la_status la_calibrate_issue(int32_t mix, int32_t mix_second, int32_t waves, int32_t workgroups, int32_t iters,
                             float *sink, void *hip_stream) {
  if (mix < 0 || mix >= MIX_COUNT || (waves != 4 && waves != 8) || workgroups < 1 || workgroups > (1 << 20) ||
      iters < 1 || !sink)
    return LA_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  if (mix_second < 0) mix_second = mix;
  if (mix_second == mix) {
    switch (mix) {
      case MIX_ADD: launch_issue<MIX_ADD, MIX_ADD>(workgroups, waves, iters, sink, st); break;
      case MIX_EXP: launch_issue<MIX_EXP, MIX_EXP>(workgroups, waves, iters, sink, st); break;
      case MIX_CVT: launch_issue<MIX_CVT, MIX_CVT>(workgroups, waves, iters, sink, st); break;
      case MIX_MFMA: launch_issue<MIX_MFMA, MIX_MFMA>(workgroups, waves, iters, sink, st); break;
      case MIX_MFMA_OPERANDS: launch_issue<MIX_MFMA_OPERANDS, MIX_MFMA_OPERANDS>(workgroups, waves, iters, sink, st); break;
      case MIX_MFMA_ADD4: launch_issue<MIX_MFMA_ADD4, MIX_MFMA_ADD4>(workgroups, waves, iters, sink, st); break;
      case MIX_MFMA_ADD8: launch_issue<MIX_MFMA_ADD8, MIX_MFMA_ADD8>(workgroups, waves, iters, sink, st); break;
      case MIX_MFMA_SOFTMAX: launch_issue<MIX_MFMA_SOFTMAX, MIX_MFMA_SOFTMAX>(workgroups, waves, iters, sink, st); break;
    }
  } else if (mix == MIX_MFMA && mix_second == MIX_ADD && waves == 8) {
    launch_issue<MIX_MFMA, MIX_ADD>(workgroups, waves, iters, sink, st);
  } else if (mix == MIX_MFMA && mix_second == MIX_EXP && waves == 8) {
    launch_issue<MIX_MFMA, MIX_EXP>(workgroups, waves, iters, sink, st);
  } else {
    return LA_ERR_UNSUPPORTED;
  }
  return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

la_status la_calibrate_read(const void *src, size_t bytes, uint32_t *sink, void *hip_stream) {
  if (!src || !sink || bytes < 16 || ((uintptr_t)src & 15)) return LA_ERR_INVALID_ARG;
  {
    ProfileScope scope(SLOT_CALIB_READ, (hipStream_t)hip_stream);
    hipLaunchKernelGGL(calib_read_kernel, dim3(256 * 16), dim3(256), 0, (hipStream_t)hip_stream, (const u32x4 *)src,
                       bytes / 16, sink);
  }
  return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

}  // extern "C"
