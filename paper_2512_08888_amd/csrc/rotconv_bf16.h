// bfloat16 storage support: bf16 tensors are widened to fp32 in the caller's workspace, the fp32
// kernels run on the copies (bf16 x bf16 products are exact in fp32 and the accumulation is fp32, so the
// arithmetic is exactly "bf16 inputs, fp32 accumulate"), and results are rounded to bf16 once, after
// the arg-max has been taken on the fp32 values.
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace rotconv {

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// round to nearest, ties to even; NaN stays NaN (quiet)
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  const uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

void launch_widen(const uint16_t* in, float* out, size_t n, hipStream_t st);
void launch_narrow(const float* in, uint16_t* out, size_t n, hipStream_t st);

}  // namespace rotconv
