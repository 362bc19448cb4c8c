// Network glue around the rotation convolution (see include/unetglue.h): streaming
// elementwise / window kernels (HBM-bound) and the GEMM-shaped layers mapped onto the
// matrix-core GEMM of glue_gemm.hip.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "glue_internal.h"
#include "rotconv.h"
#include "unetglue.h"

namespace rotconv {
namespace {

int finish() { return hipGetLastError() == hipSuccess ? ROTCONV_OK : ROTCONV_ERR_LAUNCH; }
unsigned blocks_for(size_t n) { return (unsigned)std::max<size_t>(1, std::min<size_t>((n + 255) / 256, 1u << 20)); }

typedef float f4 __attribute__((ext_vector_type(4)));

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Streaming kernels: 16 bytes per lane and access when the shapes and pointers allow (V = 4), else scalar (V = 1).
template <int V>
__global__ __launch_bounds__(256) void k_relu_fwd(const float* __restrict__ x, float* __restrict__ y, size_t n) {
  const size_t nv = n / V;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nv; i += (size_t)gridDim.x * 256) {
    if (V == 4) {
      const f4 v = reinterpret_cast<const f4*>(x)[i];
      reinterpret_cast<f4*>(y)[i] = f4{fmaxf(v[0], 0.f), fmaxf(v[1], 0.f), fmaxf(v[2], 0.f), fmaxf(v[3], 0.f)};
    } else {
      y[i] = fmaxf(x[i], 0.f);
    }
  }
  const size_t t = nv * V + (size_t)blockIdx.x * 256 + threadIdx.x;    // the last n % V elements
  if (V > 1 && t < n) y[t] = fmaxf(x[t], 0.f);
}
template <int V>
__global__ __launch_bounds__(256) void k_relu_bwd(const float* __restrict__ y, const float* __restrict__ dy,
                                                  float* __restrict__ dx, size_t n) {
  const size_t nv = n / V;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nv; i += (size_t)gridDim.x * 256) {
    if (V == 4) {
      const f4 a = reinterpret_cast<const f4*>(y)[i], d = reinterpret_cast<const f4*>(dy)[i];
      reinterpret_cast<f4*>(dx)[i] = f4{a[0] > 0.f ? d[0] : 0.f, a[1] > 0.f ? d[1] : 0.f, a[2] > 0.f ? d[2] : 0.f,
                                        a[3] > 0.f ? d[3] : 0.f};
    } else {
      dx[i] = y[i] > 0.f ? dy[i] : 0.f;
    }
  }
  const size_t t = nv * V + (size_t)blockIdx.x * 256 + threadIdx.x;
  if (V > 1 && t < n) dx[t] = y[t] > 0.f ? dy[t] : 0.f;
}

// One thread per pair of windows when V == 2 (four input columns: 16-byte row reads), else per window.
template <int V>
__global__ __launch_bounds__(256) void k_maxpool2_fwd(const float* __restrict__ x, float* __restrict__ y,
                                                      uint8_t* __restrict__ idx, size_t planes, int H, int W) {
  const int Ho = H / 2, Wo = W / 2, Wv = Wo / V;
  const size_t total = planes * Ho * Wv;
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const int ox = (int)(e % Wv) * V, oy = (int)((e / Wv) % Ho);
    const size_t pl = e / ((size_t)Wv * Ho);
    const float* p = x + (pl * H + 2 * oy) * W + 2 * ox;
    float r0[2 * V], r1[2 * V];
    if (V == 2) {
      const f4 a = *reinterpret_cast<const f4*>(p), b = *reinterpret_cast<const f4*>(p + W);
#pragma unroll
      for (int k = 0; k < 4; ++k) { r0[k] = a[k]; r1[k] = b[k]; }
    } else {
      r0[0] = p[0]; r0[1] = p[1]; r1[0] = p[W]; r1[1] = p[W + 1];
    }
    float best[V];
    int bi[V];
#pragma unroll
    for (int k = 0; k < V; ++k) {
      best[k] = r0[2 * k]; bi[k] = 0;
      if (r0[2 * k + 1] > best[k]) { best[k] = r0[2 * k + 1]; bi[k] = 1; }
      if (r1[2 * k] > best[k]) { best[k] = r1[2 * k]; bi[k] = 2; }
      if (r1[2 * k + 1] > best[k]) { best[k] = r1[2 * k + 1]; bi[k] = 3; }
    }
    const size_t o = (pl * Ho + oy) * Wo + ox;
    if (V == 2) {
      *reinterpret_cast<float2*>(y + o) = make_float2(best[0], best[V - 1]);
      *reinterpret_cast<uint16_t*>(idx + o) = (uint16_t)(bi[0] | (bi[V - 1] << 8));
    } else {
      y[o] = best[0];
      idx[o] = (uint8_t)bi[0];
    }
  }
}
// One thread per four input columns (two windows) when V == 4, else per input element.
template <int V>
__global__ __launch_bounds__(256) void k_maxpool2_bwd(const float* __restrict__ dy, const uint8_t* __restrict__ idx,
                                                      float* __restrict__ dx, size_t planes, int H, int W, int acc) {
  const int Ho = H / 2, Wo = W / 2, Wv = W / V;
  const size_t total = planes * H * Wv;
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const int xx = (int)(e % Wv) * V, yy = (int)((e / Wv) % H);
    const size_t pl = e / ((size_t)Wv * H);
    const size_t o = (pl * Ho + yy / 2) * Wo + xx / 2;
    const size_t i = (pl * H + yy) * W + xx;
    if (V == 4) {
      const float2 d = *reinterpret_cast<const float2*>(dy + o);
      const uint32_t w = *reinterpret_cast<const uint16_t*>(idx + o);
      const uint32_t r = 2 * (yy & 1);
      f4 v = f4{(w & 0xff) == r ? d.x : 0.f, (w & 0xff) == r + 1 ? d.x : 0.f, (w >> 8) == r ? d.y : 0.f,
                (w >> 8) == r + 1 ? d.y : 0.f};
      if (acc) v += *reinterpret_cast<const f4*>(dx + i);
      *reinterpret_cast<f4*>(dx + i) = v;
    } else {
      const float v = idx[o] == (uint8_t)(2 * (yy & 1) + (xx & 1)) ? dy[o] : 0.f;
      dx[i] = acc ? dx[i] + v : v;
    }
  }
}

// na, nb: elements per image of the two parts.  V == 4 needs both divisible by 4.
template <int V>
__global__ __launch_bounds__(256) void k_concat2(const float* __restrict__ a, const float* __restrict__ b,
                                                 float* __restrict__ out, int N, size_t na, size_t nb) {
  const size_t va = na / V, vb = nb / V, total = (size_t)N * (va + vb);
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const size_t n = e / (va + vb), r = e % (va + vb);
    if (V == 4) {
      reinterpret_cast<f4*>(out)[e] = r < va ? reinterpret_cast<const f4*>(a)[n * va + r]
                                             : reinterpret_cast<const f4*>(b)[n * vb + (r - va)];
    } else {
      out[e] = r < va ? a[n * va + r] : b[n * vb + (r - va)];
    }
  }
}
template <int V>
__global__ __launch_bounds__(256) void k_split2(const float* __restrict__ dcat, float* __restrict__ da,
                                                float* __restrict__ db, int N, size_t na, size_t nb, int acc) {
  const size_t va = na / V, vb = nb / V, total = (size_t)N * (va + vb);
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const size_t n = e / (va + vb), r = e % (va + vb);
    if (V == 4) {
      const f4 v = reinterpret_cast<const f4*>(dcat)[e];
      if (r < va) {
        f4* d = reinterpret_cast<f4*>(da) + (n * va + r);
        *d = acc ? *d + v : v;
      } else {
        reinterpret_cast<f4*>(db)[n * vb + (r - va)] = v;
      }
    } else {
      if (r < va) da[n * va + r] = acc ? da[n * va + r] + dcat[e] : dcat[e];
      else db[n * vb + (r - va)] = dcat[e];
    }
  }
}

// per-pixel loss into `pix`, dlogits = (softmax - onehot) * inv
__global__ __launch_bounds__(256) void k_softmax_ce(const float* __restrict__ logits, const int32_t* __restrict__ labels,
                                                    float* __restrict__ pix, float* __restrict__ dl, int N, int K,
                                                    size_t P, float inv) {
  const size_t total = (size_t)N * P;
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const size_t n = e / P, p = e % P;
    const float* lg = logits + n * K * P + p;
    float m = lg[0];
    for (int k = 1; k < K; ++k) m = fmaxf(m, lg[(size_t)k * P]);
    float s = 0.f;
    for (int k = 0; k < K; ++k) s += expf(lg[(size_t)k * P] - m);
    const int lab = labels[e];
    const bool valid = lab >= 0 && lab < K;      // a label outside 0..K-1 contributes nothing
    const float lse = m + logf(s);
    pix[e] = valid ? lse - lg[(size_t)lab * P] : 0.f;
    float* d = dl + n * K * P + p;
    for (int k = 0; k < K; ++k)
      d[(size_t)k * P] = valid ? (expf(lg[(size_t)k * P] - lse) - (k == lab ? 1.f : 0.f)) * inv : 0.f;
  }
}
// deterministic mean: 1024 threads each sum a strided subset in order, then a fixed tree
__global__ __launch_bounds__(1024) void k_mean(const float* __restrict__ v, float* __restrict__ out, size_t n, float inv) {
  __shared__ float red[1024];
  float s = 0.f;
  for (size_t i = threadIdx.x; i < n; i += 1024) s += v[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = red[0] * inv;
}

// Splits of the contraction for the weight gradients (K = pixels of one image): about 1024 workgroups,
// chunks of at least 64 pixels, at most 64 partial sums per image.
int pick_splitk(int tiles, int batch, int K) {
  int s = std::max(1, 1024 / std::max(1, tiles * batch));
  s = std::min(s, std::max(1, K / 64));
  return std::min(s, 64);
}

}  // namespace
}  // namespace rotconv

using namespace rotconv;

extern "C" {

int glue_relu_fwd(const float* x, float* y, size_t n, void* stream) {
  if (!x || !y) return ROTCONV_ERR_NULL;
  if (aligned16(x) && aligned16(y))
    hipLaunchKernelGGL(k_relu_fwd<4>, dim3(blocks_for(n / 4 + 4)), dim3(256), 0, (hipStream_t)stream, x, y, n);
  else
    hipLaunchKernelGGL(k_relu_fwd<1>, dim3(blocks_for(n)), dim3(256), 0, (hipStream_t)stream, x, y, n);
  return finish();
}
int glue_relu_bwd(const float* y, const float* dy, float* dx, size_t n, void* stream) {
  if (!y || !dy || !dx) return ROTCONV_ERR_NULL;
  if (aligned16(y) && aligned16(dy) && aligned16(dx))
    hipLaunchKernelGGL(k_relu_bwd<4>, dim3(blocks_for(n / 4 + 4)), dim3(256), 0, (hipStream_t)stream, y, dy, dx, n);
  else
    hipLaunchKernelGGL(k_relu_bwd<1>, dim3(blocks_for(n)), dim3(256), 0, (hipStream_t)stream, y, dy, dx, n);
  return finish();
}

int glue_maxpool2_fwd(const float* x, float* y, uint8_t* idx, int N, int C, int H, int W, void* stream) {
  if (!x || !y || !idx) return ROTCONV_ERR_NULL;
  if (N < 1 || C < 1 || H < 2 || W < 2 || (H & 1) || (W & 1)) return ROTCONV_ERR_SHAPE;
  const size_t planes = (size_t)N * C;
  if ((W & 3) == 0 && aligned16(x) && aligned16(y) && aligned16(idx))
    hipLaunchKernelGGL(k_maxpool2_fwd<2>, dim3(blocks_for(planes * H * W / 8)), dim3(256), 0, (hipStream_t)stream, x, y,
                       idx, planes, H, W);
  else
    hipLaunchKernelGGL(k_maxpool2_fwd<1>, dim3(blocks_for(planes * H * W / 4)), dim3(256), 0, (hipStream_t)stream, x, y,
                       idx, planes, H, W);
  return finish();
}
int glue_maxpool2_bwd(const float* dy, const uint8_t* idx, float* dx, int N, int C, int H, int W, int accumulate,
                      void* stream) {
  if (!dy || !idx || !dx) return ROTCONV_ERR_NULL;
  if (N < 1 || C < 1 || H < 2 || W < 2 || (H & 1) || (W & 1)) return ROTCONV_ERR_SHAPE;
  const size_t planes = (size_t)N * C;
  if ((W & 3) == 0 && aligned16(dy) && aligned16(dx) && aligned16(idx))
    hipLaunchKernelGGL(k_maxpool2_bwd<4>, dim3(blocks_for(planes * H * W / 4)), dim3(256), 0, (hipStream_t)stream, dy,
                       idx, dx, planes, H, W, accumulate);
  else
    hipLaunchKernelGGL(k_maxpool2_bwd<1>, dim3(blocks_for(planes * H * W)), dim3(256), 0, (hipStream_t)stream, dy, idx,
                       dx, planes, H, W, accumulate);
  return finish();
}

size_t glue_upconv2_workspace_bytes(int N, int Cin, int Cout, int H, int W) {
  const int tiles = ((Cin + 127) / 128) * ((4 * Cout + 127) / 128);
  return (size_t)N * pick_splitk(tiles, N, H * W) * Cin * 4 * Cout * sizeof(float);
}
int glue_upconv2_fwd(const float* x, const float* w, float* y, int N, int Cin, int Cout, int H, int W, void* stream) {
  if (!x || !w || !y) return ROTCONV_ERR_NULL;
  if (N < 1 || Cin < 1 || Cout < 1 || H < 1 || W < 1) return ROTCONV_ERR_SHAPE;
  GemmArgs a{};
  a.M = 4 * Cout; a.N = H * W; a.K = Cin; a.lda = 4 * Cout; a.ldb = H * W; a.ldc = H * W; a.transA = 1; a.transB = 0;
  a.batch = N; a.splitk = 1; a.strideA = 0; a.strideB = (size_t)Cin * H * W; a.strideC = (size_t)Cout * 4 * H * W;
  a.shufB = 0; a.shufC = 1; a.shufH = H; a.shufW = W;
  launch_gemm(a, w, x, y, (hipStream_t)stream);
  return finish();
}
int glue_upconv2_bwd_data(const float* dy, const float* w, float* dx, int N, int Cin, int Cout, int H, int W,
                          void* stream) {
  if (!dy || !w || !dx) return ROTCONV_ERR_NULL;
  if (N < 1 || Cin < 1 || Cout < 1 || H < 1 || W < 1) return ROTCONV_ERR_SHAPE;
  GemmArgs a{};
  a.M = Cin; a.N = H * W; a.K = 4 * Cout; a.lda = 4 * Cout; a.ldb = 0; a.ldc = H * W; a.transA = 0; a.transB = 0;
  a.batch = N; a.splitk = 1; a.strideA = 0; a.strideB = (size_t)Cout * 4 * H * W; a.strideC = (size_t)Cin * H * W;
  a.shufB = 1; a.shufC = 0; a.shufH = H; a.shufW = W;
  launch_gemm(a, w, dy, dx, (hipStream_t)stream);
  return finish();
}
int glue_upconv2_bwd_weight(const float* x, const float* dy, float* dw, int N, int Cin, int Cout, int H, int W,
                            void* ws, size_t ws_bytes, void* stream) {
  if (!x || !dy || !dw) return ROTCONV_ERR_NULL;
  if (N < 1 || Cin < 1 || Cout < 1 || H < 1 || W < 1) return ROTCONV_ERR_SHAPE;
  if (!ws || ws_bytes < glue_upconv2_workspace_bytes(N, Cin, Cout, H, W)) return ROTCONV_ERR_WORKSPACE;
  const int tiles = ((Cin + 127) / 128) * ((4 * Cout + 127) / 128);
  GemmArgs a{};
  a.M = Cin; a.N = 4 * Cout; a.K = H * W; a.lda = H * W; a.ldb = 0; a.ldc = 4 * Cout; a.transA = 0; a.transB = 1;
  a.batch = N; a.splitk = pick_splitk(tiles, N, H * W); a.strideA = (size_t)Cin * H * W;
  a.strideB = (size_t)Cout * 4 * H * W; a.strideC = (size_t)Cin * 4 * Cout;
  a.shufB = 1; a.shufC = 0; a.shufH = H; a.shufW = W;
  launch_gemm(a, x, dy, (float*)ws, (hipStream_t)stream);
  launch_sum_parts((const float*)ws, dw, a.strideC, N * a.splitk, a.strideC, (hipStream_t)stream);
  return finish();
}

int glue_concat2(const float* a, const float* b, float* out, int N, int Ca, int Cb, size_t P, void* stream) {
  if (!a || !b || !out) return ROTCONV_ERR_NULL;
  if (N < 1 || Ca < 1 || Cb < 1 || P < 1) return ROTCONV_ERR_SHAPE;
  const size_t na = (size_t)Ca * P, nb = (size_t)Cb * P;
  if (na % 4 == 0 && nb % 4 == 0 && aligned16(a) && aligned16(b) && aligned16(out))
    hipLaunchKernelGGL(k_concat2<4>, dim3(blocks_for((size_t)N * (na + nb) / 4)), dim3(256), 0, (hipStream_t)stream, a, b,
                       out, N, na, nb);
  else
    hipLaunchKernelGGL(k_concat2<1>, dim3(blocks_for((size_t)N * (na + nb))), dim3(256), 0, (hipStream_t)stream, a, b, out,
                       N, na, nb);
  return finish();
}
int glue_split2(const float* dcat, float* da, float* db, int N, int Ca, int Cb, size_t P, int accumulate_a,
                void* stream) {
  if (!dcat || !da || !db) return ROTCONV_ERR_NULL;
  if (N < 1 || Ca < 1 || Cb < 1 || P < 1) return ROTCONV_ERR_SHAPE;
  const size_t na = (size_t)Ca * P, nb = (size_t)Cb * P;
  if (na % 4 == 0 && nb % 4 == 0 && aligned16(dcat) && aligned16(da) && aligned16(db))
    hipLaunchKernelGGL(k_split2<4>, dim3(blocks_for((size_t)N * (na + nb) / 4)), dim3(256), 0, (hipStream_t)stream, dcat,
                       da, db, N, na, nb, accumulate_a);
  else
    hipLaunchKernelGGL(k_split2<1>, dim3(blocks_for((size_t)N * (na + nb))), dim3(256), 0, (hipStream_t)stream, dcat, da,
                       db, N, na, nb, accumulate_a);
  return finish();
}

size_t glue_conv1x1_workspace_bytes(int N, int Cin, int Cout, size_t P) {
  const int tiles = ((Cout + 127) / 128) * ((Cin + 127) / 128);
  return (size_t)N * pick_splitk(tiles, N, (int)P) * Cout * Cin * sizeof(float);
}
int glue_conv1x1_fwd(const float* x, const float* w, float* y, int N, int Cin, int Cout, size_t P, void* stream) {
  if (!x || !w || !y) return ROTCONV_ERR_NULL;
  if (N < 1 || Cin < 1 || Cout < 1 || P < 1 || P > 0x7fffffff) return ROTCONV_ERR_SHAPE;
  GemmArgs a{};
  a.M = Cout; a.N = (int)P; a.K = Cin; a.lda = Cin; a.ldb = (int)P; a.ldc = (int)P; a.batch = N; a.splitk = 1;
  a.strideB = (size_t)Cin * P; a.strideC = (size_t)Cout * P;
  launch_gemm(a, w, x, y, (hipStream_t)stream);
  return finish();
}
int glue_conv1x1_bwd_data(const float* dy, const float* w, float* dx, int N, int Cin, int Cout, size_t P,
                          void* stream) {
  if (!dy || !w || !dx) return ROTCONV_ERR_NULL;
  if (N < 1 || Cin < 1 || Cout < 1 || P < 1 || P > 0x7fffffff) return ROTCONV_ERR_SHAPE;
  GemmArgs a{};
  a.M = Cin; a.N = (int)P; a.K = Cout; a.lda = Cin; a.transA = 1; a.ldb = (int)P; a.ldc = (int)P; a.batch = N;
  a.splitk = 1; a.strideB = (size_t)Cout * P; a.strideC = (size_t)Cin * P;
  launch_gemm(a, w, dy, dx, (hipStream_t)stream);
  return finish();
}
int glue_conv1x1_bwd_weight(const float* x, const float* dy, float* dw, int N, int Cin, int Cout, size_t P, void* ws,
                            size_t ws_bytes, void* stream) {
  if (!x || !dy || !dw) return ROTCONV_ERR_NULL;
  if (N < 1 || Cin < 1 || Cout < 1 || P < 1 || P > 0x7fffffff) return ROTCONV_ERR_SHAPE;
  if (!ws || ws_bytes < glue_conv1x1_workspace_bytes(N, Cin, Cout, P)) return ROTCONV_ERR_WORKSPACE;
  const int tiles = ((Cout + 127) / 128) * ((Cin + 127) / 128);
  GemmArgs a{};
  a.M = Cout; a.N = Cin; a.K = (int)P; a.lda = (int)P; a.ldb = (int)P; a.transB = 1; a.ldc = Cin; a.batch = N;
  a.splitk = pick_splitk(tiles, N, (int)P); a.strideA = (size_t)Cout * P; a.strideB = (size_t)Cin * P;
  a.strideC = (size_t)Cout * Cin;
  launch_gemm(a, dy, x, (float*)ws, (hipStream_t)stream);
  launch_sum_parts((const float*)ws, dw, a.strideC, N * a.splitk, a.strideC, (hipStream_t)stream);
  return finish();
}

int glue_softmax_ce(const float* logits, const int32_t* labels, float* loss, float* dlogits, int N, int K, size_t P,
                    void* ws, size_t ws_bytes, void* stream) {
  if (!logits || !labels || !loss || !dlogits) return ROTCONV_ERR_NULL;
  if (N < 1 || K < 1 || P < 1) return ROTCONV_ERR_SHAPE;
  if (!ws || ws_bytes < (size_t)N * P * sizeof(float)) return ROTCONV_ERR_WORKSPACE;
  const float inv = 1.0f / (float)((double)N * (double)P);
  hipLaunchKernelGGL(k_softmax_ce, dim3(blocks_for((size_t)N * P)), dim3(256), 0, (hipStream_t)stream, logits, labels,
                     (float*)ws, dlogits, N, K, P, inv);
  hipLaunchKernelGGL(k_mean, dim3(1), dim3(1024), 0, (hipStream_t)stream, (const float*)ws, loss, (size_t)N * P, inv);
  return finish();
}

}  // extern "C"
