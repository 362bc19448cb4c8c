// Staging kernels: bf16 <-> fp32 conversion (HBM-bound streaming, 8 elements per lane) and row re-pitch.
#include "rotconv_bf16.h"

#include <algorithm>

namespace rotconv {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_widen(const uint16_t* __restrict__ in, float* __restrict__ out, size_t n,
                                               int vec) {
  const size_t n8 = vec ? n / 8 : 0;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
    const u4 v = reinterpret_cast<const u4*>(in)[i];
    f4 a, b;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      a[2 * k] = __uint_as_float(v[k] << 16);
      a[2 * k + 1] = __uint_as_float(v[k] & 0xffff0000u);
      b[2 * k] = __uint_as_float(v[2 + k] << 16);
      b[2 * k + 1] = __uint_as_float(v[2 + k] & 0xffff0000u);
    }
    reinterpret_cast<f4*>(out)[2 * i] = a;
    reinterpret_cast<f4*>(out)[2 * i + 1] = b;
  }
  for (size_t i = n8 * 8 + (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
    out[i] = bf16_to_f32(in[i]);
}

__global__ __launch_bounds__(256) void k_narrow(const float* __restrict__ in, uint16_t* __restrict__ out, size_t n,
                                                int vec) {
  const size_t n8 = vec ? n / 8 : 0;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
    const f4 a = reinterpret_cast<const f4*>(in)[2 * i], b = reinterpret_cast<const f4*>(in)[2 * i + 1];
    u4 v;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      v[k] = (uint32_t)f32_to_bf16(a[2 * k]) | ((uint32_t)f32_to_bf16(a[2 * k + 1]) << 16);
      v[2 + k] = (uint32_t)f32_to_bf16(b[2 * k]) | ((uint32_t)f32_to_bf16(b[2 * k + 1]) << 16);
    }
    reinterpret_cast<u4*>(out)[i] = v;
  }
  for (size_t i = n8 * 8 + (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
    out[i] = f32_to_bf16(in[i]);
}

// Row re-pitch: dst rows of Wd elements from src rows of Ws elements; columns beyond Ws get `fill` (Wd < Ws: crop).
template <typename T>
__global__ __launch_bounds__(256) void k_repitch(const T* __restrict__ src, T* __restrict__ dst, size_t rows, int Ws,
                                                 int Wd, T fill) {
  const size_t total = rows * (size_t)Wd;
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const size_t r = e / Wd;
    const int c = (int)(e - r * Wd);
    dst[e] = c < Ws ? src[r * Ws + c] : fill;
  }
}

unsigned blocks_for(size_t n) { return (unsigned)std::max<size_t>(1, std::min<size_t>((n / 8 + 255) / 256, 1u << 16)); }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

void launch_widen(const uint16_t* in, float* out, size_t n, hipStream_t st) {
  hipLaunchKernelGGL(k_widen, dim3(blocks_for(n)), dim3(256), 0, st, in, out, n, aligned16(in) && aligned16(out) ? 1 : 0);
}
void launch_narrow(const float* in, uint16_t* out, size_t n, hipStream_t st) {
  hipLaunchKernelGGL(k_narrow, dim3(blocks_for(n)), dim3(256), 0, st, in, out, n, aligned16(in) && aligned16(out) ? 1 : 0);
}

void launch_repitch(const void* src, void* dst, size_t rows, int Ws, int Wd, int elem_bytes, uint32_t fill,
                    hipStream_t st) {
  const size_t total = rows * (size_t)Wd;
  const unsigned blocks = (unsigned)std::max<size_t>(1, std::min<size_t>((total + 255) / 256, 1u << 16));
  if (elem_bytes == 1)
    hipLaunchKernelGGL(k_repitch<uint8_t>, dim3(blocks), dim3(256), 0, st, static_cast<const uint8_t*>(src),
                       static_cast<uint8_t*>(dst), rows, Ws, Wd, (uint8_t)fill);
  else if (elem_bytes == 2)
    hipLaunchKernelGGL(k_repitch<uint16_t>, dim3(blocks), dim3(256), 0, st, static_cast<const uint16_t*>(src),
                       static_cast<uint16_t*>(dst), rows, Ws, Wd, (uint16_t)fill);
  else
    hipLaunchKernelGGL(k_repitch<uint32_t>, dim3(blocks), dim3(256), 0, st, static_cast<const uint32_t*>(src),
                       static_cast<uint32_t*>(dst), rows, Ws, Wd, fill);
}

}  // namespace rotconv
