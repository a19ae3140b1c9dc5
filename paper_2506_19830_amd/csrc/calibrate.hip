// Two calibration kernels for the benchmark (not part of the verification path): what this very chip reaches on a
// pure bf16 MFMA loop and on a pure streaming read, so that a roofline fraction can be quoted against the
// achievable rate next to the published peak.
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
