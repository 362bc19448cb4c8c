// Internal declarations of the network-glue kernels (see include/unetglue.h).
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace rotconv {

struct GemmArgs {
  int M, N, K;
  int lda, ldb, ldc;
  int transA, transB;       // A stored [K][M] / B stored [N][K]
  int batch, splitk;        // grid.z = batch * splitk; output z at C + z*strideC
  size_t strideA, strideB;  // per batch
  size_t strideC;           // per (batch, split)
  int shufB, shufC;         // B is read / C is written through the 2x2 pixel-shuffle map
  int shufH, shufW;         // input extent (H, W) of that map
  int bf16A, bf16B, bf16C;  // the operand holds bfloat16 (widened on load / rounded on store) instead of fp32
};

void launch_gemm(const GemmArgs& a, const void* A, const void* B, void* C, hipStream_t st);
void launch_sum_parts(const float* part, float* out, size_t n, int nparts, size_t stride, hipStream_t st);

}  // namespace rotconv
