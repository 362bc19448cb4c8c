// Generic fp32 GEMM on the matrix cores for the network glue around the rotation
// convolution (2x2 transposed-convolution up-sampling, 1x1 head): C = op(A) * op(B),
// optionally batched and/or split along K with an ordered reduction afterwards.
// 128 x 128 x 16 tiles, four waves of 64 x 64 (sixteen 16x16x4 MFMA accumulators each),
// operands staged through LDS k-major so both fragment reads are conflict-free,
// next tile prefetched into registers while the current one is multiplied.
#include <hip/hip_runtime.h>

#include "glue_internal.h"
#include "rotconv_bf16.h"

namespace rotconv {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 16, PITCH = 144, NT = 256;

// Address of element (r, p) of the virtual matrix T[(co,a,b)][(h,w)] = y[co][2h+a][2w+b] that a 2x2
// stride-2 transposed convolution reads / writes (r = 4 co + 2 a + b, p = h W + w, y is [Cout][2H][2W]).
__device__ __forceinline__ size_t shuffled(int r, int p, int H, int W) {
  const int co = r >> 2, a = (r >> 1) & 1, b = r & 1, h = p / W, w = p - h * W;
  return ((size_t)co * 2 * H + 2 * h + a) * (2 * W) + 2 * w + b;
}

// A element (m, k): transA ? A[k*lda + m] : A[m*lda + k];  B element (k, n): transB ? B[n*ldb + k] : B[k*ldb + n]
template <bool TA, bool TB>
__global__ __launch_bounds__(NT) void k_gemm(const void* __restrict__ A, const void* __restrict__ B,
                                            void* __restrict__ C, GemmArgs p) {
  __shared__ float As[2][BK][PITCH];
  __shared__ float Bs[2][BK][PITCH];
  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, lg = lane / 16, lc = lane % 16;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int z = blockIdx.z;
  const int batch = z / p.splitk, ks = z % p.splitk;
  const int kchunk = ((p.K + p.splitk - 1) / p.splitk + BK - 1) / BK * BK;
  const int kbeg = ks * kchunk, kend = min(p.K, kbeg + kchunk);
  const size_t Abase = (size_t)batch * p.strideA, Bbase = (size_t)batch * p.strideB, Cbase = (size_t)z * p.strideC;
  // element access in the operand's storage type (wave-uniform choice)
  auto ldA = [&](size_t off) {
    return p.bf16A ? bf16_to_f32(static_cast<const uint16_t*>(A)[Abase + off]) : static_cast<const float*>(A)[Abase + off];
  };
  auto ldB = [&](size_t off) {
    return p.bf16B ? bf16_to_f32(static_cast<const uint16_t*>(B)[Bbase + off]) : static_cast<const float*>(B)[Bbase + off];
  };

  float ra[8], rb[8];
  auto gload = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int m, k;
      if (TA) { m = tid % 128; k = tid / 128 + 2 * i; } else { k = tid % 16; m = tid / 16 + 16 * i; }
      const int gm = m0 + m, gk = k0 + k;
      const bool ok = gm < p.M && gk < kend;
      const size_t off = TA ? (size_t)gk * p.lda + gm : (size_t)gm * p.lda + gk;
      ra[i] = ok ? ldA(off) : 0.f;
      int n, kb;
      if (TB) { kb = tid % 16; n = tid / 16 + 16 * i; } else { n = tid % 128; kb = tid / 128 + 2 * i; }
      const int gn = n0 + n, gkb = k0 + kb;
      const bool okb = gn < p.N && gkb < kend;
      size_t offb = TB ? (size_t)gn * p.ldb + gkb : (size_t)gkb * p.ldb + gn;
      if (p.shufB) offb = shuffled(TB ? gn : gkb, TB ? gkb : gn, p.shufH, p.shufW);
      rb[i] = okb ? ldB(offb) : 0.f;
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int m, k;
      if (TA) { m = tid % 128; k = tid / 128 + 2 * i; } else { k = tid % 16; m = tid / 16 + 16 * i; }
      As[buf][k][m] = ra[i];
      int n, kb;
      if (TB) { kb = tid % 16; n = tid / 16 + 16 * i; } else { n = tid % 128; kb = tid / 128 + 2 * i; }
      Bs[buf][kb][n] = rb[i];
    }
  };

  f4 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f4{0.f, 0.f, 0.f, 0.f};
  const int wm = (wave / 2) * 64, wn = (wave % 2) * 64;

  if (kbeg < kend) {
    gload(kbeg);
    sstore(0);
    __syncthreads();
    int buf = 0;
    for (int k0 = kbeg; k0 < kend; k0 += BK) {
      const bool more = k0 + BK < kend;
      if (more) gload(k0 + BK);
#pragma unroll
      for (int kk = 0; kk < BK; kk += 4) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = As[buf][kk + lg][wm + i * 16 + lc];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = Bs[buf][kk + lg][wn + j * 16 + lc];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i], b[j], acc[i][j], 0, 0, 0);
      }
      if (more) sstore(buf ^ 1);
      __syncthreads();
      buf ^= 1;
    }
  }
  // accumulator tile (i, j): rows m = wm + 16 i + 4 lg + r, column n = wn + 16 j + lc
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int gm = m0 + wm + 16 * i + 4 * lg + r, gn = n0 + wn + 16 * j + lc;
        if (gm < p.M && gn < p.N) {
          const size_t off = Cbase + (p.shufC ? shuffled(gm, gn, p.shufH, p.shufW) : (size_t)gm * p.ldc + gn);
          if (p.bf16C) static_cast<uint16_t*>(C)[off] = f32_to_bf16(acc[i][j][r]);
          else static_cast<float*>(C)[off] = acc[i][j][r];
        }
      }
}

// out[e] = sum_z part[z][e], z ascending (fixed order).
__global__ __launch_bounds__(256) void k_sum_parts(const float* __restrict__ part, float* __restrict__ out, size_t n,
                                                   int nparts, size_t stride) {
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= n) return;
  float s = 0.f;
  for (int zz = 0; zz < nparts; ++zz) s += part[(size_t)zz * stride + e];
  out[e] = s;
}

}  // namespace

void launch_gemm(const GemmArgs& a, const void* A, const void* B, void* C, hipStream_t st) {
  dim3 grid((a.M + BM - 1) / BM, (a.N + BN - 1) / BN, a.batch * a.splitk);
  if (a.transA && a.transB) hipLaunchKernelGGL((k_gemm<true, true>), grid, dim3(NT), 0, st, A, B, C, a);
  else if (a.transA) hipLaunchKernelGGL((k_gemm<true, false>), grid, dim3(NT), 0, st, A, B, C, a);
  else if (a.transB) hipLaunchKernelGGL((k_gemm<false, true>), grid, dim3(NT), 0, st, A, B, C, a);
  else hipLaunchKernelGGL((k_gemm<false, false>), grid, dim3(NT), 0, st, A, B, C, a);
}

void launch_sum_parts(const float* part, float* out, size_t n, int nparts, size_t stride, hipStream_t st) {
  hipLaunchKernelGGL(k_sum_parts, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part, out, n, nparts, stride);
}

}  // namespace rotconv
