// Regularisers of the steerable filter pair (paper Sec. III-D, Eq. 18-20): magnitude matching and
// orthogonality of the two base banks, with their gradients.  One workgroup per filter reduces
// ||wx||^2, ||wy||^2 and <wx, wy> in a fixed tree and writes that filter's gradient; a second, single
// workgroup adds the per-filter terms in ascending order.  HBM-bound: w is read twice, dw written once.
#include <hip/hip_runtime.h>

#include "rotconv.h"

namespace rotconv {
namespace {

__device__ __forceinline__ float block_sum(float v, float* red) {
  const int t = threadIdx.x;
  __syncthreads();
  red[t] = v;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (t < w) red[t] += red[t + w];
    __syncthreads();
  }
  return red[0];
}

__global__ __launch_bounds__(256) void k_steer_reg(const float* __restrict__ w, int Cout, int per, float lmag,
                                                   float lorth, float eps, float* __restrict__ terms,
                                                   float* __restrict__ dw, int accumulate) {
  __shared__ float red[256];
  const int b = blockIdx.x;
  const float* wx = w + (size_t)b * per;
  const float* wy = w + ((size_t)Cout + b) * per;
  float sx = 0.f, sy = 0.f, sd = 0.f;
  for (int i = threadIdx.x; i < per; i += 256) {
    const float a = wx[i], c = wy[i];
    sx += a * a; sy += c * c; sd += a * c;
  }
  const float nx2 = block_sum(sx, red), ny2 = block_sum(sy, red), dot = block_sum(sd, red);
  const float nx = sqrtf(nx2), ny = sqrtf(ny2);
  const float diff = nx - ny;                       // Eq. 19 term: diff^2
  const float den = nx * ny + eps;
  const float c = dot / den;                        // Eq. 20 term: c^2
  if (threadIdx.x == 0) { terms[2 * b] = diff * diff; terms[2 * b + 1] = c * c; }
  if (!dw) return;
  const float invB = 1.0f / (float)Cout;
  // d diff^2 / d wx = 2 diff wx / nx,  d diff^2 / d wy = -2 diff wy / ny
  const float mx = nx > 0.f ? 2.f * diff / nx : 0.f, my = ny > 0.f ? -2.f * diff / ny : 0.f;
  // d c / d wx = wy / den - dot ny (wx / nx) / den^2, likewise for wy
  const float kx = nx > 0.f ? dot * ny / (nx * den * den) : 0.f, ky = ny > 0.f ? dot * nx / (ny * den * den) : 0.f;
  float* dx = dw + (size_t)b * per;
  float* dy = dw + ((size_t)Cout + b) * per;
  for (int i = threadIdx.x; i < per; i += 256) {
    const float a = wx[i], v = wy[i];
    const float gx = invB * (lmag * mx * a + lorth * 2.f * c * (v / den - kx * a));
    const float gy = invB * (lmag * my * v + lorth * 2.f * c * (a / den - ky * v));
    dx[i] = accumulate ? dx[i] + gx : gx;
    dy[i] = accumulate ? dy[i] + gy : gy;
  }
}

__global__ __launch_bounds__(256) void k_steer_reg_sum(const float* __restrict__ terms, int Cout,
                                                       float* __restrict__ losses) {
  __shared__ float red[256];
  float m = 0.f, o = 0.f;
  for (int b = threadIdx.x; b < Cout; b += 256) { m += terms[2 * b]; o += terms[2 * b + 1]; }
  const float sm = block_sum(m, red), so = block_sum(o, red);
  if (threadIdx.x == 0) { losses[0] = sm / (float)Cout; losses[1] = so / (float)Cout; }
}

}  // namespace
}  // namespace rotconv

extern "C" int rotconv_steerable_reg(const float* w, int32_t Cout, int32_t per, float lambda_mag, float lambda_orth,
                                     float eps, float* losses, float* dw, int32_t accumulate, void* ws, size_t ws_bytes,
                                     void* stream) {
  if (!w || !losses) return ROTCONV_ERR_NULL;
  if (Cout < 1 || per < 1) return ROTCONV_ERR_SHAPE;
  if (!ws || ws_bytes < (size_t)Cout * 2 * sizeof(float)) return ROTCONV_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* terms = static_cast<float*>(ws);
  hipLaunchKernelGGL(rotconv::k_steer_reg, dim3(Cout), dim3(256), 0, st, w, Cout, per, lambda_mag, lambda_orth, eps,
                     terms, dw, accumulate);
  hipLaunchKernelGGL(rotconv::k_steer_reg_sum, dim3(1), dim3(256), 0, st, terms, Cout, losses);
  return hipGetLastError() == hipSuccess ? ROTCONV_OK : ROTCONV_ERR_LAUNCH;
}
