// GEMMs on the matrix cores for the network glue around the rotation convolution (2x2
// transposed-convolution up-sampling, 1x1 head): C = op(A) * op(B), optionally batched and/or
// split along K with an ordered reduction afterwards.  Two kernels of the same shape, 128 x 128
// tiles, four waves of 64 x 64 (sixteen accumulators each), operands staged through LDS, the next
// tile prefetched into registers while the current one is multiplied:
//   k_gemm    fp32 operands, 16x16x4 fp32 instruction, 16-deep tiles, LDS k-major;
//   k_gemm16  bfloat16 operands, 16x16x32 bf16 instruction (fp32 accumulation), 32-deep tiles,
//             LDS row-major with the contraction index contiguous.
#include <hip/hip_runtime.h>

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
template <bool TA, bool TB>
__global__ __launch_bounds__(NT) void k_gemm(const float* __restrict__ A, const float* __restrict__ B,
                                            float* __restrict__ C, GemmArgs p) {
  __shared__ float As[2][BK][PITCH];
  __shared__ float Bs[2][BK][PITCH];
  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, lg = lane / 16, lc = lane % 16;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int z = blockIdx.z;
  const int batch = z / p.splitk, ks = z % p.splitk;
  const int kchunk = ((p.K + p.splitk - 1) / p.splitk + BK - 1) / BK * BK;
  const int kbeg = ks * kchunk, kend = min(p.K, kbeg + kchunk);
  const size_t Abase = (size_t)batch * p.strideA, Bbase = (size_t)batch * p.strideB, Cbase = (size_t)z * p.strideC;
  // a fetched element is zeroed outside the matrix only when it is written to LDS, after the current tile's
  // multiplications: nothing between a load and that point waits for it
  const float* Ap = A + Abase;
  const float* Bp = B + Bbase;

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

  float ra[8], rb[8];
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
      As[buf][k][m] = (aok[i] && k0 + k < kend) ? ra[i] : 0.f;
      int n, kb;
      if (TB) { kb = tid % 16; n = tid / 16 + 16 * i; } else { n = tid % 128; kb = tid / 128 + 2 * i; }
      Bs[buf][kb][n] = (bok[i] && k0 + kb < kend) ? rb[i] : 0.f;
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
          C[off] = acc[i][j][r];
        }
      }
  }
}

// The same product for bfloat16 operands on the bf16 matrix instruction (16 x 16 x 32, fp32 accumulation; result
// fp32 or rounded to bfloat16).  128 x 128 x 32 tiles; LDS holds both operands row-major with the contraction
// index contiguous (pitch 40 halfwords: the sixteen 16-byte fragment reads of a quarter wave fall into distinct
// banks), so a fragment is one ds_read_b128.  Element (row, k) of a tile is fetched by thread
//   k-major storage (TA / !TB):   row = tid % 128, k = 16 (tid / 128) + i   (lanes along the row: coalesced; the
//                                 thread's sixteen k are packed and written as two 16-byte LDS stores)
//   row-major storage (!TA / TB): row = tid / 32 + 8 i, k = tid % 32        (lanes along k: coalesced)
// for i = 0 .. 15; every offset is the thread's base plus a multiple of a launch constant.
constexpr int BK16 = 32, PITCH16 = 40;
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

template <bool TA, bool TB, bool OUT16>
__global__ __launch_bounds__(NT) void k_gemm16(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B,
                                              void* __restrict__ C, GemmArgs p) {
  __shared__ __attribute__((aligned(16))) uint16_t As[2][BM][PITCH16];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN][PITCH16];
  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, lg = lane / 16, lc = lane % 16;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int z = blockIdx.z;
  const int batch = z / p.splitk, ks = z % p.splitk;
  const int kchunk = ((p.K + p.splitk - 1) / p.splitk + BK16 - 1) / BK16 * BK16;
  const int kbeg = ks * kchunk, kend = min(p.K, kbeg + kchunk);
  const uint16_t* Ap = A + (size_t)batch * p.strideA;
  const uint16_t* Bp = B + (size_t)batch * p.strideB;
  const size_t Cbase = (size_t)z * p.strideC;
  constexpr bool AKM = TA, BKM = !TB;   // operand stored k-major
  const int t128 = tid % 128, h128 = tid / 128, t32 = tid % 32, h32 = tid / 32;

  // A: thread's base offset and what element i adds; rows at and beyond arow_end lie outside the matrix
  const size_t abase = AKM ? (size_t)(16 * h128) * p.lda + m0 + t128 : (size_t)(m0 + h32) * p.lda + t32;
  const size_t ai = AKM ? (size_t)p.lda : (size_t)8 * p.lda;
  const int arow = AKM ? m0 + t128 : m0 + h32;     // row of element 0 (k-major: of every element)
  // B, plain: as A.  Through the pixel-shuffle map, T[r][pix] sits at shuf_row(r) + shuf_pix(pix):
  //   TB  (row n = r, k = pixel): base shuf_row(n0 + h32), element i adds i * shuf_row(8); the tile adds shuf_pix(k)
  //   !TB (row n = pixel, k = r = k0 + 16 h128 + i, k0 % 32 == 0): base shuf_pix(n) + shuf_row(16 h128), element i
  //        adds shuf_row(i) (taken apart at compile time), the tile adds shuf_row(k0)
  const int brow = BKM ? n0 + t128 : n0 + h32;
  const size_t plane = (size_t)4 * p.shufH * p.shufW;   // one output channel of the shuffled tensor = shuf_row(4)
  size_t bbase, bi;
  if (p.shufB) {
    bbase = BKM ? (brow < p.N ? shuf_pix(brow, p.shufW) : 0) + 4 * h128 * plane : shuf_row(min(brow, p.N - 1), p.shufH, p.shufW);
    bi = BKM ? 0 : 2 * plane;
  } else {
    bbase = BKM ? (size_t)(16 * h128) * p.ldb + brow : (size_t)brow * p.ldb + t32;
    bi = BKM ? (size_t)p.ldb : (size_t)8 * p.ldb;
  }

  uint16_t ra[16], rb[16];
  auto a_in = [&](int i, int k0) { return AKM ? (arow < p.M && k0 + 16 * h128 + i < kend) : (arow + 8 * i < p.M && k0 + t32 < kend); };
  auto b_in = [&](int i, int k0) { return BKM ? (brow < p.N && k0 + 16 * h128 + i < kend) : (brow + 8 * i < p.N && k0 + t32 < kend); };
  auto gload = [&](int k0) {
    const size_t astep = AKM ? (size_t)k0 * p.lda : (size_t)k0;
    size_t bstep;
    if (p.shufB) bstep = BKM ? (size_t)(k0 / 4) * plane : shuf_pix(k0 + t32 < kend ? k0 + t32 : kbeg, p.shufW);
    else bstep = BKM ? (size_t)k0 * p.ldb : (size_t)k0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      ra[i] = Ap[a_in(i, k0) ? abase + astep + i * ai : 0];
      size_t bo = bbase + bstep + i * bi;
      if (p.shufB && BKM) bo += (size_t)(i / 4) * plane + (size_t)((i / 2) % 2) * 2 * p.shufW + i % 2;
      rb[i] = Bp[b_in(i, k0) ? bo : 0];
    }
  };
  auto put = [&](uint16_t (*T)[PITCH16], const uint16_t* r, bool kmajor, auto inside) {
    if (kmajor) {
      uint32_t w[8];
#pragma unroll
      for (int i = 0; i < 8; ++i)
        w[i] = (inside(2 * i) ? (uint32_t)r[2 * i] : 0u) | ((inside(2 * i + 1) ? (uint32_t)r[2 * i + 1] : 0u) << 16);
      u4* d = reinterpret_cast<u4*>(&T[t128][16 * h128]);
      d[0] = u4{w[0], w[1], w[2], w[3]};
      d[1] = u4{w[4], w[5], w[6], w[7]};
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) T[h32 + 8 * i][t32] = inside(i) ? r[i] : (uint16_t)0;
    }
  };
  auto sstore = [&](int buf, int k0) {
    put(As[buf], ra, AKM, [&](int i) { return a_in(i, k0); });
    put(Bs[buf], rb, BKM, [&](int i) { return b_in(i, k0); });
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
    for (int k0 = kbeg; k0 < kend; k0 += BK16) {
      const bool more = k0 + BK16 < kend;
      if (more) gload(k0 + BK16);
      __builtin_amdgcn_sched_barrier(0);
      bf8 a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = *reinterpret_cast<const bf8*>(&As[buf][wm + 16 * i + lc][8 * lg]);
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = *reinterpret_cast<const bf8*>(&Bs[buf][wn + 16 * j + lc][8 * lg]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (more) sstore(buf ^ 1, k0 + BK16);
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
          if (OUT16) static_cast<uint16_t*>(C)[off] = f32_to_bf16(acc[i][j][r]);
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

void launch_gemm_f32(const GemmArgs& a, const void* A, const void* B, void* C, hipStream_t st) {
  dim3 grid((a.M + BM - 1) / BM, (a.N + BN - 1) / BN, a.batch * a.splitk);
  const float* Af = static_cast<const float*>(A);
  const float* Bf = static_cast<const float*>(B);
  float* Cf = static_cast<float*>(C);
  if (a.transA && a.transB) hipLaunchKernelGGL((k_gemm<true, true>), grid, dim3(NT), 0, st, Af, Bf, Cf, a);
  else if (a.transA) hipLaunchKernelGGL((k_gemm<true, false>), grid, dim3(NT), 0, st, Af, Bf, Cf, a);
  else if (a.transB) hipLaunchKernelGGL((k_gemm<false, true>), grid, dim3(NT), 0, st, Af, Bf, Cf, a);
  else hipLaunchKernelGGL((k_gemm<false, false>), grid, dim3(NT), 0, st, Af, Bf, Cf, a);
}
template <bool OUT16>
void launch_gemm_bf16(const GemmArgs& a, const void* A, const void* B, void* C, hipStream_t st) {
  dim3 grid((a.M + BM - 1) / BM, (a.N + BN - 1) / BN, a.batch * a.splitk);
  const uint16_t* A16 = static_cast<const uint16_t*>(A);
  const uint16_t* B16 = static_cast<const uint16_t*>(B);
  if (a.transA && a.transB) hipLaunchKernelGGL((k_gemm16<true, true, OUT16>), grid, dim3(NT), 0, st, A16, B16, C, a);
  else if (a.transA) hipLaunchKernelGGL((k_gemm16<true, false, OUT16>), grid, dim3(NT), 0, st, A16, B16, C, a);
  else if (a.transB) hipLaunchKernelGGL((k_gemm16<false, true, OUT16>), grid, dim3(NT), 0, st, A16, B16, C, a);
  else hipLaunchKernelGGL((k_gemm16<false, false, OUT16>), grid, dim3(NT), 0, st, A16, B16, C, a);
}
void launch_gemm(const GemmArgs& a, const void* A, const void* B, void* C, hipStream_t st) {
  // the glue uses three storage combinations: all fp32, bf16 operands with an fp32 or a bf16 result
  if (a.bf16A && a.bf16B && a.bf16C) launch_gemm_bf16<true>(a, A, B, C, st);
  else if (a.bf16A && a.bf16B) launch_gemm_bf16<false>(a, A, B, C, st);
  else launch_gemm_f32(a, A, B, C, st);
}

void launch_sum_parts(const float* part, float* out, size_t n, int nparts, size_t stride, hipStream_t st) {
  hipLaunchKernelGGL(k_sum_parts, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part, out, n, nparts, stride);
}

}  // namespace rotconv
