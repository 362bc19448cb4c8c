// Network glue around the rotation convolution (see include/unetglue.h): streaming
// elementwise / window kernels (HBM-bound) and the GEMM-shaped layers mapped onto the
// matrix-core GEMM of glue_gemm.hip.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "glue_internal.h"
#include "rotconv.h"
#include "unetglue.h"

namespace rotconv {
namespace {

int finish() { return hipGetLastError() == hipSuccess ? ROTCONV_OK : ROTCONV_ERR_LAUNCH; }
unsigned blocks_for(size_t n) { return (unsigned)std::min<size_t>((n + 255) / 256, 1u << 20); }

__global__ __launch_bounds__(256) void k_relu_fwd(const float* __restrict__ x, float* __restrict__ y, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) y[i] = fmaxf(x[i], 0.f);
}
__global__ __launch_bounds__(256) void k_relu_bwd(const float* __restrict__ y, const float* __restrict__ dy,
                                                  float* __restrict__ dx, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
    dx[i] = y[i] > 0.f ? dy[i] : 0.f;
}

__global__ __launch_bounds__(256) void k_maxpool2_fwd(const float* __restrict__ x, float* __restrict__ y,
                                                      uint8_t* __restrict__ idx, size_t planes, int H, int W) {
  const int Ho = H / 2, Wo = W / 2;
  const size_t total = planes * Ho * Wo;
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const int ox = (int)(e % Wo), oy = (int)((e / Wo) % Ho);
    const size_t pl = e / ((size_t)Wo * Ho);
    const float* p = x + (pl * H + 2 * oy) * W + 2 * ox;
    float best = p[0];
    int bi = 0;
    if (p[1] > best) { best = p[1]; bi = 1; }
    if (p[W] > best) { best = p[W]; bi = 2; }
    if (p[W + 1] > best) { best = p[W + 1]; bi = 3; }
    y[e] = best;
    idx[e] = (uint8_t)bi;
  }
}
__global__ __launch_bounds__(256) void k_maxpool2_bwd(const float* __restrict__ dy, const uint8_t* __restrict__ idx,
                                                      float* __restrict__ dx, size_t planes, int H, int W, int acc) {
  const size_t total = planes * H * W;
  const int Ho = H / 2, Wo = W / 2;
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const int xx = (int)(e % W), yy = (int)((e / W) % H);
    const size_t pl = e / ((size_t)W * H);
    const size_t o = (pl * Ho + yy / 2) * Wo + xx / 2;
    const float v = idx[o] == (uint8_t)(2 * (yy & 1) + (xx & 1)) ? dy[o] : 0.f;
    dx[e] = acc ? dx[e] + v : v;
  }
}

__global__ __launch_bounds__(256) void k_concat2(const float* __restrict__ a, const float* __restrict__ b,
                                                 float* __restrict__ out, int N, size_t na, size_t nb) {
  const size_t total = (size_t)N * (na + nb);
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const size_t n = e / (na + nb), r = e % (na + nb);
    out[e] = r < na ? a[n * na + r] : b[n * nb + (r - na)];
  }
}
__global__ __launch_bounds__(256) void k_split2(const float* __restrict__ dcat, float* __restrict__ da,
                                                float* __restrict__ db, int N, size_t na, size_t nb, int acc) {
  const size_t total = (size_t)N * (na + nb);
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const size_t n = e / (na + nb), r = e % (na + nb);
    if (r < na) da[n * na + r] = acc ? da[n * na + r] + dcat[e] : dcat[e];
    else db[n * nb + (r - na)] = dcat[e];
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
  hipLaunchKernelGGL(k_relu_fwd, dim3(blocks_for(n)), dim3(256), 0, (hipStream_t)stream, x, y, n);
  return finish();
}
int glue_relu_bwd(const float* y, const float* dy, float* dx, size_t n, void* stream) {
  if (!y || !dy || !dx) return ROTCONV_ERR_NULL;
  hipLaunchKernelGGL(k_relu_bwd, dim3(blocks_for(n)), dim3(256), 0, (hipStream_t)stream, y, dy, dx, n);
  return finish();
}

int glue_maxpool2_fwd(const float* x, float* y, uint8_t* idx, int N, int C, int H, int W, void* stream) {
  if (!x || !y || !idx) return ROTCONV_ERR_NULL;
  if (N < 1 || C < 1 || H < 2 || W < 2 || (H & 1) || (W & 1)) return ROTCONV_ERR_SHAPE;
  const size_t planes = (size_t)N * C;
  hipLaunchKernelGGL(k_maxpool2_fwd, dim3(blocks_for(planes * H * W / 4)), dim3(256), 0, (hipStream_t)stream, x, y, idx,
                     planes, H, W);
  return finish();
}
int glue_maxpool2_bwd(const float* dy, const uint8_t* idx, float* dx, int N, int C, int H, int W, int accumulate,
                      void* stream) {
  if (!dy || !idx || !dx) return ROTCONV_ERR_NULL;
  if (N < 1 || C < 1 || H < 2 || W < 2 || (H & 1) || (W & 1)) return ROTCONV_ERR_SHAPE;
  const size_t planes = (size_t)N * C;
  hipLaunchKernelGGL(k_maxpool2_bwd, dim3(blocks_for(planes * H * W)), dim3(256), 0, (hipStream_t)stream, dy, idx, dx,
                     planes, H, W, accumulate);
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
  hipLaunchKernelGGL(k_concat2, dim3(blocks_for((size_t)N * (Ca + Cb) * P)), dim3(256), 0, (hipStream_t)stream, a, b, out,
                     N, (size_t)Ca * P, (size_t)Cb * P);
  return finish();
}
int glue_split2(const float* dcat, float* da, float* db, int N, int Ca, int Cb, size_t P, int accumulate_a,
                void* stream) {
  if (!dcat || !da || !db) return ROTCONV_ERR_NULL;
  if (N < 1 || Ca < 1 || Cb < 1 || P < 1) return ROTCONV_ERR_SHAPE;
  hipLaunchKernelGGL(k_split2, dim3(blocks_for((size_t)N * (Ca + Cb) * P)), dim3(256), 0, (hipStream_t)stream, dcat, da,
                     db, N, (size_t)Ca * P, (size_t)Cb * P, accumulate_a);
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
