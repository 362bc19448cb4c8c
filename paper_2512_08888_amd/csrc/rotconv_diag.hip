// Two measuring kernels for the benchmark's "measured peak" figures (not on the hot path): a register-resident
// loop of independent matrix instructions, and a plain 16-byte-per-lane copy.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "rotconv.h"

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));

// Eight independent accumulator tiles per wave, n_iter rounds; operands never change, nothing touches memory until
// the end (the sum of the tiles goes to sink so that the loop is not removed).
__global__ __launch_bounds__(256) void k_diag_mfma_f32(float* sink, int n_iter) {
  f4 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = f4{0.f, 0.f, 0.f, 0.f};
  const float a = 1.0f + (float)(threadIdx.x & 3) * 0.25f, b = 0.5f;
  for (int it = 0; it < n_iter; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[i], 0, 0, 0);
  }
  f4 s = acc[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) s += acc[i];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s[0] + s[1] + s[2] + s[3];
}

__global__ __launch_bounds__(256) void k_diag_mfma_bf16(float* sink, int n_iter) {
  f4 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = f4{0.f, 0.f, 0.f, 0.f};
  bf8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(1.0f + (float)((threadIdx.x + i) & 3) * 0.25f); b[i] = (__bf16)0.5f; }
  for (int it = 0; it < n_iter; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
  }
  f4 s = acc[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) s += acc[i];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s[0] + s[1] + s[2] + s[3];
}

__global__ __launch_bounds__(256) void k_diag_copy(f4* __restrict__ dst, const f4* __restrict__ src, size_t n4) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

constexpr int kDiagBlocks = 256 * 8;     // eight workgroups of four waves per compute unit

}  // namespace

extern "C" {

size_t rotconv_diag_mfma_sink_bytes(void) { return (size_t)kDiagBlocks * 256 * sizeof(float); }

int rotconv_diag_mfma(int dtype, int n_iter, float* sink, void* stream, double* flops) {
  if (!sink || n_iter < 1) return ROTCONV_ERR_NULL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const double waves = (double)kDiagBlocks * 4.0;
  if (dtype == ROTCONV_F32) {
    hipLaunchKernelGGL(k_diag_mfma_f32, dim3(kDiagBlocks), dim3(256), 0, st, sink, n_iter);
    if (flops) *flops = waves * n_iter * 8.0 * (2.0 * 16 * 16 * 4);
  } else if (dtype == ROTCONV_BF16) {
    hipLaunchKernelGGL(k_diag_mfma_bf16, dim3(kDiagBlocks), dim3(256), 0, st, sink, n_iter);
    if (flops) *flops = waves * n_iter * 8.0 * (2.0 * 16 * 16 * 32);
  } else {
    return ROTCONV_ERR_UNSUPPORTED;
  }
  return hipGetLastError() == hipSuccess ? ROTCONV_OK : ROTCONV_ERR_LAUNCH;
}

int rotconv_diag_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src) return ROTCONV_ERR_NULL;
  if (bytes % 16 || reinterpret_cast<uintptr_t>(dst) % 16 || reinterpret_cast<uintptr_t>(src) % 16) return ROTCONV_ERR_SHAPE;
  hipLaunchKernelGGL(k_diag_copy, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(stream), static_cast<f4*>(dst),
                     static_cast<const f4*>(src), bytes / 16);
  return hipGetLastError() == hipSuccess ? ROTCONV_OK : ROTCONV_ERR_LAUNCH;
}

}  // extern "C"
