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

// Packed routing of two bf16 values by their arg-max indices (max-pool backward, Eq. 12): x16 holds the two
// idx bytes as halfwords, rs2 the wanted orientation in both halfwords; returns 0xffff in each halfword whose idx
// matches, else 0 (halfword-wise min(x ^ r, 1) - 1).
__device__ __forceinline__ uint32_t match_mask2(uint32_t x16, uint32_t rs2) {
  const uint32_t y = x16 ^ rs2, one2 = 0x00010001u;
  uint32_t t, m;
  asm("v_pk_min_u16 %0, %1, %2" : "=v"(t) : "v"(y), "s"(one2));
  asm("v_pk_sub_u16 %0, %1, %2" : "=v"(m) : "v"(t), "s"(one2));
  return m;
}

void launch_widen(const uint16_t* in, float* out, size_t n, hipStream_t st);
void launch_narrow(const float* in, uint16_t* out, size_t n, hipStream_t st);
// rows of Ws elements (1, 2 or 4 bytes each) -> rows of Wd elements; new columns are filled with `fill`
void launch_repitch(const void* src, void* dst, size_t rows, int Ws, int Wd, int elem_bytes, uint32_t fill,
                    hipStream_t st);

}  // namespace rotconv
