// Generic fp32 GEMM on the matrix cores for the network glue around the rotation
// convolution (2x2 transposed-convolution up-sampling, 1x1 head): C = op(A) * op(B),
// optionally batched and/or split along K with an ordered reduction afterwards.
// 128 x 128 x 16 tiles, four waves of 64 x 64 (sixteen 16x16x4 MFMA accumulators each),
// operands staged through LDS k-major so both fragment reads are conflict-free,
// next tile prefetched into registers while the current one is multiplied.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "glue_internal.h"
#include "rotconv_bf16.h"

namespace rotconv {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 16, PITCH = 144, NT = 256;

// The virtual matrix T[(co,a,b)][(h,w)] = y[co][2h+a][2w+b] that a 2x2 stride-2 transposed convolution reads /
// writes (r = 4 co + 2 a + b, p = h W + w, y is [Cout][2H][2W]): address = row part (r) + pixel part (p).
__device__ __forceinline__ size_t shuf_row(int r, int H, int W) {
  const int co = r >> 2, a = (r >> 1) & 1, b = r & 1;
  return ((size_t)co * 2 * H + a) * (2 * W) + b;
}
__device__ __forceinline__ size_t shuf_pix(int p, int W) {
  const int h = p / W, w = p - h * W;
  return (size_t)(2 * h) * (2 * W) + 2 * w;
}

// A element (m, k): transA ? A[k*lda + m] : A[m*lda + k];  B element (k, n): transB ? B[n*ldb + k] : B[k*ldb + n].
// Every thread fetches eight A and eight B elements per 16-deep tile; the parts of their addresses that do not
// depend on the tile (row / column, pixel-shuffle terms, bounds) are computed once, so a tile costs additions only.
// BF: 0 = fp32 operands and result; 1 = bfloat16 A and B, fp32 result (weight gradients); 2 = all three bfloat16.
// (compile-time, so that a tile's sixteen loads are issued back to back instead of one per branch)
template <bool TA, bool TB, int BF>
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
  // a fetched element as it sits in memory; widened (and zeroed outside the matrix) only when it is written to
  // LDS, after the current tile's multiplications: nothing between a load and that point waits for it
  using Raw = typename std::conditional<BF != 0, uint16_t, float>::type;
  const Raw* Ap = static_cast<const Raw*>(A) + Abase;
  const Raw* Bp = static_cast<const Raw*>(B) + Bbase;
  auto widen = [](Raw v) -> float {
    if constexpr (BF != 0) return bf16_to_f32(v);
    else return v;
  };

  // tile-independent parts.  A: element i is (m, k) = TA ? (tid % 128, tid / 128 + 2 i) : (tid / 16 + 16 i, tid % 16);
  // B: element i is (n, k) = TB ? (tid / 16 + 16 i, tid % 16) : (tid % 128, tid / 128 + 2 i).
  size_t aoff[8], boff[8];
  bool aok[8], bok[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int m = TA ? tid % 128 : tid / 16 + 16 * i, k = TA ? tid / 128 + 2 * i : tid % 16;
    const int gm = m0 + m;
    aok[i] = gm < p.M;
    aoff[i] = aok[i] ? (TA ? (size_t)k * p.lda + gm : (size_t)gm * p.lda + k) : 0;
    const int n = TB ? tid / 16 + 16 * i : tid % 128, kb = TB ? tid % 16 : tid / 128 + 2 * i;
    const int gn = n0 + n;
    bok[i] = gn < p.N;
    if (!bok[i]) boff[i] = 0;
    else if (p.shufB) boff[i] = TB ? shuf_row(gn, p.shufH, p.shufW)                       // + pixel part of k, per tile
                                   : shuf_pix(gn, p.shufW) + shuf_row(kb, p.shufH, p.shufW);  // + row part of k0, per tile
    else boff[i] = TB ? (size_t)gn * p.ldb + kb : (size_t)kb * p.ldb + gn;
  }

  Raw ra[8], rb[8];
  auto gload = [&](int k0) {
    // what the tile adds to the offsets (k0 is a multiple of 16, so with shufB and !TB the row part of k0 + kb
    // is the sum of the two row parts: k0's low bits are zero)
    const size_t astep = TA ? (size_t)k0 * p.lda : (size_t)k0;
    size_t bstep;
    if (p.shufB) bstep = TB ? shuf_pix(k0 + tid % 16 < kend ? k0 + tid % 16 : kbeg, p.shufW) : shuf_row(k0, p.shufH, p.shufW);
    else bstep = TB ? (size_t)k0 : (size_t)k0 * p.ldb;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      // every load is issued (from element 0 of the operand where the element lies outside the matrix): a load
      // under a branch would be waited for before the next one is issued
      const int k = TA ? tid / 128 + 2 * i : tid % 16;
      ra[i] = Ap[(aok[i] && k0 + k < kend) ? aoff[i] + astep : 0];
      const int kb = TB ? tid % 16 : tid / 128 + 2 * i;
      rb[i] = Bp[(bok[i] && k0 + kb < kend) ? boff[i] + bstep : 0];
    }
  };
  auto sstore = [&](int buf, int k0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int m, k;
      if (TA) { m = tid % 128; k = tid / 128 + 2 * i; } else { k = tid % 16; m = tid / 16 + 16 * i; }
      As[buf][k][m] = (aok[i] && k0 + k < kend) ? widen(ra[i]) : 0.f;
      int n, kb;
      if (TB) { kb = tid % 16; n = tid / 16 + 16 * i; } else { n = tid % 128; kb = tid / 128 + 2 * i; }
      Bs[buf][kb][n] = (bok[i] && k0 + kb < kend) ? widen(rb[i]) : 0.f;
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
    sstore(0, kbeg);
    __syncthreads();
    int buf = 0;
    for (int k0 = kbeg; k0 < kend; k0 += BK) {
      const bool more = k0 + BK < kend;
      if (more) gload(k0 + BK);
      __builtin_amdgcn_sched_barrier(0);
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
      __builtin_amdgcn_sched_barrier(0);
      if (more) sstore(buf ^ 1, k0 + BK);
      __syncthreads();
      buf ^= 1;
    }
  }
  // accumulator tile (i, j): rows m = wm + 16 i + 4 lg + r, column n = wn + 16 j + lc
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int gn = n0 + wn + 16 * j + lc;
    if (gn >= p.N) continue;
    const size_t coff = Cbase + (p.shufC ? shuf_pix(gn, p.shufW) : (size_t)gn);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int gm = m0 + wm + 16 * i + 4 * lg + r;
        if (gm < p.M) {
          const size_t off = coff + (p.shufC ? shuf_row(gm, p.shufH, p.shufW) : (size_t)gm * p.ldc);
          if (BF == 2) static_cast<uint16_t*>(C)[off] = f32_to_bf16(acc[i][j][r]);
          else static_cast<float*>(C)[off] = acc[i][j][r];
        }
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

template <int BF>
void launch_gemm_t(const GemmArgs& a, const void* A, const void* B, void* C, hipStream_t st) {
  dim3 grid((a.M + BM - 1) / BM, (a.N + BN - 1) / BN, a.batch * a.splitk);
  if (a.transA && a.transB) hipLaunchKernelGGL((k_gemm<true, true, BF>), grid, dim3(NT), 0, st, A, B, C, a);
  else if (a.transA) hipLaunchKernelGGL((k_gemm<true, false, BF>), grid, dim3(NT), 0, st, A, B, C, a);
  else if (a.transB) hipLaunchKernelGGL((k_gemm<false, true, BF>), grid, dim3(NT), 0, st, A, B, C, a);
  else hipLaunchKernelGGL((k_gemm<false, false, BF>), grid, dim3(NT), 0, st, A, B, C, a);
}
void launch_gemm(const GemmArgs& a, const void* A, const void* B, void* C, hipStream_t st) {
  // the glue uses three storage combinations: all fp32, bf16 operands with an fp32 or a bf16 result
  if (a.bf16A && a.bf16B && a.bf16C) launch_gemm_t<2>(a, A, B, C, st);
  else if (a.bf16A && a.bf16B) launch_gemm_t<1>(a, A, B, C, st);
  else launch_gemm_t<0>(a, A, B, C, st);
}

void launch_sum_parts(const float* part, float* out, size_t n, int nparts, size_t stride, hipStream_t st) {
  hipLaunchKernelGGL(k_sum_parts, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part, out, n, nparts, stride);
}

}  // namespace rotconv
