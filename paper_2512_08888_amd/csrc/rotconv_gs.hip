// Matrix-multiply + scatter family (fp32) for the layers the register-resident kernels do not take (k != 3,
// stride != 1, pad != 1, and the unfused gradient calls): the two-step organisation of the paper's Sec. IV on the
// matrix cores.
//
//   forward   P[(q,co,u)][pixel] = sum_ci F_q[co,ci,u] X[ci,pixel]        one GEMM per image, M = Q Cout k^2
//             Y_r[co,yo,xo] = sum_u P[(q,co,u)][yo s + i - pad, xo s + j - pad],  (i,j) = where quarter turn s_r puts
//             base tap u (Eq. 8), then max / arg-max over the pool group (Eq. 10)      -- the scatter, as a gather
//   gradients D[(q,co,u)][pixel] = sum_s Delta_(q,s)[co, (y + pad - i)/s, (x + pad - j)/s]   (Eq. 12 routed, or a dense dy)
//             dX = F^T D (one GEMM per image, Eq. 13/15);  dF = D X^T (one GEMM per image, split along the pixels,
//             parts added in order, Eq. 14/16), then the transposed first-quadrant expansion.
//
// The products / routed gradients of a few images at a time live in the workspace (k^2 Q Cout H W floats per image).
// The multiplications are shared by the quarter turns exactly as in the register-resident kernels; what this family
// gives up is their on-chip placement: every product goes through memory once.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>

#include "glue_internal.h"
#include "rotconv_bf16.h"
#include "rotconv_gs.h"

namespace rotconv {
namespace {

struct GsGeom {
  int N, Cin, H, W, Cout, k, kk, R, Q, ng, stride, pad, Ho, Wo, relu;
};

GsGeom gs_geom(const rotconv_plan* p) {
  GsGeom g;
  g.N = p->d.N; g.Cin = p->d.Cin; g.H = p->d.H; g.W = p->d.W; g.Cout = p->d.Cout; g.k = p->d.k; g.kk = p->kk;
  g.R = p->d.R; g.Q = p->host.Q; g.ng = p->ng; g.stride = p->d.stride; g.pad = p->d.pad; g.Ho = p->Ho; g.Wo = p->Wo;
  g.relu = 0;
  return g;
}

size_t align256(size_t v) { return (v + 255) / 256 * 256; }

// base bank(s) -> the GEMM operand [(q, co, u)][ci] (first-quadrant banks, Sec. III-D / Eq. 17); one thread per
// (q, co, ci), its k^2 taps read the same base filter.
__global__ __launch_bounds__(256) void k_gs_pack(const float* __restrict__ w, float* __restrict__ a,
                                                 const int32_t* __restrict__ fq_src, const float* __restrict__ fq_coef,
                                                 const double* __restrict__ fq_coef64, int Q, int Cout, int Cin, int kk,
                                                 int round16) {
  const int total = Q * Cout * Cin;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int ci = e % Cin, co = (e / Cin) % Cout, q = e / (Cin * Cout);
  const size_t slices = (size_t)Cout * Cin;
  const float* src = w + ((size_t)co * Cin + ci) * kk;
  for (int u = 0; u < kk; ++u) {
    float acc = 0.f;
    if (round16) {    // bf16 plans: the combination in fp64, rounded to fp32 and to bf16 once each
      double a64 = 0.0;
      for (int z = 0; z < kMaxNnz; ++z) {
        const int s = fq_src[(q * kk + u) * kMaxNnz + z];
        if (s >= 0) a64 += fq_coef64[(q * kk + u) * kMaxNnz + z] * (double)src[(size_t)(s / kk) * slices * kk + s % kk];
      }
      acc = bf16_to_f32(f32_to_bf16((float)a64));
    } else {
#pragma unroll
      for (int z = 0; z < kMaxNnz; ++z) {
        const int s = fq_src[(q * kk + u) * kMaxNnz + z];
        if (s >= 0) acc += fq_coef[(q * kk + u) * kMaxNnz + z] * src[(size_t)(s / kk) * slices * kk + s % kk];
      }
    }
    a[((size_t)(q * Cout + co) * kk + u) * Cin + ci] = acc;
  }
}

constexpr int kMaxKK = 225;      // k <= 15

// Forward placement (Eq. 8) as a gather over the products of `nb` images, then Eq. 10.  One thread per output pixel
// of a pooled channel (FUSED) or of a filter (all its orientations are written).  The tap offsets of the four
// quarter turns sit in LDS; a product outside the image is read from a valid address and dropped.
template <bool FUSED>
__global__ __launch_bounds__(256) void k_gs_place(const float* __restrict__ P, const int32_t* __restrict__ rq_of_r,
                                                  const int32_t* __restrict__ turn_tap, float* __restrict__ yout,
                                                  uint8_t* __restrict__ idx, GsGeom g, int n0) {
  __shared__ int siy[4 * kMaxKK], six[4 * kMaxKK];
  for (int i = threadIdx.x; i < 4 * g.kk; i += 256) {
    const int t = turn_tap[i];
    siy[i] = t / g.k - g.pad;
    six[i] = t % g.k - g.pad;
  }
  __syncthreads();
  const int Po = g.Ho * g.Wo, Pi = g.H * g.W;
  const int p = blockIdx.x * 256 + threadIdx.x;
  if (p >= Po) return;
  const int oy = (p / g.Wo) * g.stride, ox = (p % g.Wo) * g.stride;
  const int b = blockIdx.z, n = n0 + b;
  const int rstep = FUSED ? g.ng : 1;
  const float* Pb = P + (size_t)b * g.Q * g.Cout * g.kk * Pi;
  const int nchan = FUSED ? g.Cout * g.ng : g.Cout;
  for (int chan = blockIdx.y; chan < nchan; chan += gridDim.y) {
    const int co = FUSED ? chan / g.ng : chan, grp = FUSED ? chan % g.ng : 0;
    float best = 0.f;
    int best_r = -1;
    for (int r = grp; r < g.R; r += rstep) {
      const int rq = rq_of_r[r], q = rq >> 2, s = rq & 3;
      const float* Pq = Pb + (size_t)(q * g.Cout + co) * g.kk * Pi;
      const int* ty = siy + s * g.kk;
      const int* tx = six + s * g.kk;
      float acc = 0.f;
#pragma unroll 4
      for (int u = 0; u < g.kk; ++u) {
        const int yi = oy + ty[u], xi = ox + tx[u];
        const bool ok = (unsigned)yi < (unsigned)g.H && (unsigned)xi < (unsigned)g.W;
        const float v = Pq[(size_t)u * Pi + (ok ? yi * g.W + xi : 0)];
        acc += ok ? v : 0.f;
      }
      if (FUSED) {
        if (best_r < 0 || acc > best) { best = acc; best_r = r; }
      } else {
        yout[(((size_t)n * g.Cout + co) * g.R + r) * Po + p] = acc;
      }
    }
    if (FUSED) {
      const size_t o = ((size_t)n * g.Cout * g.ng + chan) * Po + p;
      const bool dead = g.relu && !(best > 0.f);
      yout[o] = dead ? 0.f : best;
      idx[o] = dead ? (uint8_t)255 : (uint8_t)best_r;
    }
  }
}

// D[(q,co,u)][input pixel] of `nb` images: the gradient reaching input pixel (y, x) through base tap u of bank q,
// summed over the bank's quarter turns.  ROUTED: from the pooled gradient and idx (Eq. 12); else from a dense dy.
// One thread per input pixel of a (bank, filter): it walks the k^2 taps, whose sources lie in a k x k neighbourhood
// per quarter turn (offsets in LDS); sources outside the output map are read from a valid address and dropped, so
// no load waits for a compare.  S1: stride 1 (no divisibility tests).
template <bool ROUTED, bool S1>
__global__ __launch_bounds__(256) void k_gs_route(const float* __restrict__ gsrc, const uint8_t* __restrict__ idx,
                                                  const int32_t* __restrict__ rot_of,
                                                  const int32_t* __restrict__ turn_tap, float* __restrict__ D, GsGeom g,
                                                  int n0) {
  __shared__ int sdy[4 * kMaxKK], sdx[4 * kMaxKK];
  for (int i = threadIdx.x; i < 4 * g.kk; i += 256) {
    const int t = turn_tap[i];
    sdy[i] = g.pad - t / g.k;
    sdx[i] = g.pad - t % g.k;
  }
  __syncthreads();
  const int Po = g.Ho * g.Wo, Pi = g.H * g.W;
  const int p = blockIdx.x * 256 + threadIdx.x;
  if (p >= Pi) return;
  const int y = p / g.W, x = p % g.W;
  const int b = blockIdx.z, n = n0 + b;
  const int QC = g.Q * g.Cout;
  for (int qc = blockIdx.y; qc < QC; qc += gridDim.y) {      // qc = q * Cout + co
    const int co = qc % g.Cout, q = qc / g.Cout;
    int rot[4];
    const float* gp[4];
    const uint8_t* ip[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      rot[s] = rot_of[q * 4 + s];
      const int r = max(rot[s], 0);
      const size_t plane = ROUTED ? (((size_t)n * g.Cout + co) * g.ng + r % g.ng) * Po
                                  : (((size_t)n * g.Cout + co) * g.R + r) * Po;
      gp[s] = gsrc + plane;
      ip[s] = ROUTED ? idx + plane : nullptr;
    }
    float* Dq = D + ((size_t)b * QC + qc) * g.kk * Pi + p;
#pragma unroll 2
    for (int u = 0; u < g.kk; ++u) {
      float acc = 0.f;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        if (rot[s] < 0) continue;
        const int ny = y + sdy[s * g.kk + u], nx = x + sdx[s * g.kk + u];
        int oy = ny, ox = nx;
        bool ok = true;
        if (!S1) {
          oy = ny / g.stride; ox = nx / g.stride;
          ok = ny >= 0 && nx >= 0 && oy * g.stride == ny && ox * g.stride == nx;
        }
        ok = ok && (unsigned)oy < (unsigned)g.Ho && (unsigned)ox < (unsigned)g.Wo;
        const int o = ok ? oy * g.Wo + ox : 0;
        const float gv = gp[s][o];
        if (ROUTED) ok = ok && ip[s][o] == rot[s];
        acc += ok ? gv : 0.f;
      }
      Dq[(size_t)u * Pi] = acc;
    }
  }
}

// acc[e] = (first ? 0 : acc[e]) + sum of the parts, ascending.
__global__ __launch_bounds__(256) void k_gs_sum_acc(const float* __restrict__ part, float* __restrict__ acc, size_t n,
                                                    int nparts, int first) {
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= n) return;
  float s = first ? 0.f : acc[e];
  for (int z = 0; z < nparts; ++z) s += part[(size_t)z * n + e];
  acc[e] = s;
}

// dw[b][co][ci][t] = sum over the transposed first-quadrant expansion's row (b, t) of coef * dF[(q, co, u)][ci]
// (Eq. 16 / the chain rule through Eq. 17), fixed order.
__global__ __launch_bounds__(256) void k_gs_reduce_w(const float* __restrict__ dF, float* __restrict__ dw,
                                                     const int32_t* __restrict__ ptr, const int32_t* __restrict__ col,
                                                     const float* __restrict__ coef, int B, int Cout, int Cin, int kk) {
  const int total = B * Cout * Cin;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int ci = e % Cin, co = (e / Cin) % Cout, b = e / (Cin * Cout);
  for (int t = 0; t < kk; ++t) {
    float acc = 0.f;
    for (int z = ptr[b * kk + t]; z < ptr[b * kk + t + 1]; ++z) {
      const int q = col[z] / kk, u = col[z] % kk;
      acc += coef[z] * dF[((size_t)(q * Cout + co) * kk + u) * Cin + ci];
    }
    dw[(((size_t)b * Cout + co) * Cin + ci) * kk + t] = acc;
  }
}

// images whose products / routed gradients are held at once: at most 512 MiB of them, at least one image
int chunk_images(const rotconv_plan* p) {
  const double per = 4.0 * p->host.Q * p->d.Cout * p->kk * p->d.H * p->d.W;
  return (int)std::max(1.0, std::min((double)p->d.N, (double)p->gs_chunk_bytes / per));
}

// split of the weight gradient's pixel contraction: enough workgroups to fill the chip, at least 256 pixels each
int bwdw_splitk(const rotconv_plan* p, int nb) {
  const int M = p->host.Q * p->d.Cout * p->kk;
  const long tiles = (long)((M + 127) / 128) * ((p->d.Cin + 127) / 128) * nb;
  const long want = (768 + tiles - 1) / tiles;
  const long cap = std::max(1, p->d.H * p->d.W / 256);
  return (int)std::max(1L, std::min({want, cap, 64L}));
}

struct GsLayout { size_t a, pd, part, dF, total; };
GsLayout gs_layout(const rotconv_plan* p) {
  const size_t M = (size_t)p->host.Q * p->d.Cout * p->kk;
  const int nb = chunk_images(p);
  GsLayout L;
  L.a = 0;
  L.pd = align256(M * p->d.Cin * 4);
  L.part = L.pd + align256((size_t)nb * M * p->d.H * p->d.W * 4);
  L.dF = L.part + align256((size_t)nb * bwdw_splitk(p, nb) * M * p->d.Cin * 4);
  L.total = L.dF + align256(M * p->d.Cin * 4);
  return L;
}

void pack(const rotconv_plan* p, const float* w, float* a, hipStream_t st) {
  const int total = p->host.Q * p->d.Cout * p->d.Cin;
  hipLaunchKernelGGL(k_gs_pack, dim3((total + 255) / 256), dim3(256), 0, st, w, a, p->dev.fq_src, p->dev.fq_coef,
                     p->dev.fq_coef64,
                     p->host.Q, p->d.Cout, p->d.Cin, p->kk, p->d.dtype == ROTCONV_BF16 ? 1 : 0);
}

GemmArgs gemm_args() {
  GemmArgs a{};
  a.batch = 1; a.splitk = 1;
  return a;
}

void forward(const rotconv_plan* p, bool fused, const float* x, const float* w, float* yout, uint8_t* idx, void* ws,
             hipStream_t st) {
  GsGeom g = gs_geom(p);
  g.relu = fused && p->d.activation == ROTCONV_ACT_RELU;
  const GsLayout L = gs_layout(p);
  char* c = static_cast<char*>(ws);
  float* A = reinterpret_cast<float*>(c + L.a);
  float* P = reinterpret_cast<float*>(c + L.pd);
  pack(p, w, A, st);
  const int M = g.Q * g.Cout * g.kk, Pi = g.H * g.W, Po = g.Ho * g.Wo;
  const int nbmax = chunk_images(p);
  for (int n0 = 0; n0 < g.N; n0 += nbmax) {
    const int nb = std::min(nbmax, g.N - n0);
    GemmArgs a = gemm_args();
    a.M = M; a.N = Pi; a.K = g.Cin; a.lda = g.Cin; a.ldb = Pi; a.ldc = Pi;
    a.batch = nb; a.strideA = 0; a.strideB = (size_t)g.Cin * Pi; a.strideC = (size_t)M * Pi;
    launch_gemm(a, A, x + (size_t)n0 * g.Cin * Pi, P, st);
    dim3 grid((Po + 255) / 256, std::min(fused ? g.Cout * g.ng : g.Cout, 65535), nb);
    if (fused) hipLaunchKernelGGL(k_gs_place<true>, grid, dim3(256), 0, st, P, p->dev.rq_of_r, p->dev.turn_tap, yout, idx, g, n0);
    else hipLaunchKernelGGL(k_gs_place<false>, grid, dim3(256), 0, st, P, p->dev.rq_of_r, p->dev.turn_tap, yout, idx, g, n0);
  }
}

void route(const rotconv_plan* p, const GsGeom& g, bool routed, const float* gsrc, const uint8_t* idx, float* D, int n0,
           int nb, hipStream_t st) {
  dim3 grid((g.H * g.W + 255) / 256, std::min(g.Q * g.Cout, 65535), nb);
  const bool s1 = g.stride == 1;
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, grid, dim3(256), 0, st, gsrc, idx, p->dev.rot_of, p->dev.turn_tap, D, g, n0);
  };
  if (routed) { if (s1) go(k_gs_route<true, true>); else go(k_gs_route<true, false>); }
  else { if (s1) go(k_gs_route<false, true>); else go(k_gs_route<false, false>); }
}

void backward_data(const rotconv_plan* p, bool routed, const float* gsrc, const uint8_t* idx, const float* w, float* dx,
                   void* ws, hipStream_t st) {
  const GsGeom g = gs_geom(p);
  const GsLayout L = gs_layout(p);
  char* c = static_cast<char*>(ws);
  float* A = reinterpret_cast<float*>(c + L.a);
  float* D = reinterpret_cast<float*>(c + L.pd);
  pack(p, w, A, st);
  const int M = g.Q * g.Cout * g.kk, Pi = g.H * g.W;
  const int nbmax = chunk_images(p);
  for (int n0 = 0; n0 < g.N; n0 += nbmax) {
    const int nb = std::min(nbmax, g.N - n0);
    route(p, g, routed, gsrc, idx, D, n0, nb, st);
    GemmArgs a = gemm_args();             // dX[ci][pixel] = sum_m A[m][ci] D[m][pixel]
    a.M = g.Cin; a.N = Pi; a.K = M; a.transA = 1; a.lda = g.Cin; a.ldb = Pi; a.ldc = Pi;
    a.batch = nb; a.strideA = 0; a.strideB = (size_t)M * Pi; a.strideC = (size_t)g.Cin * Pi;
    launch_gemm(a, A, D, dx + (size_t)n0 * g.Cin * Pi, st);
  }
}

void backward_weight(const rotconv_plan* p, bool routed, const float* x, const float* gsrc, const uint8_t* idx,
                     float* dw, void* ws, hipStream_t st) {
  const GsGeom g = gs_geom(p);
  const GsLayout L = gs_layout(p);
  char* c = static_cast<char*>(ws);
  float* D = reinterpret_cast<float*>(c + L.pd);
  float* part = reinterpret_cast<float*>(c + L.part);
  float* dF = reinterpret_cast<float*>(c + L.dF);
  const int M = g.Q * g.Cout * g.kk, Pi = g.H * g.W;
  const int nbmax = chunk_images(p);
  const int sk = bwdw_splitk(p, nbmax);
  const size_t nF = (size_t)M * g.Cin;
  for (int n0 = 0; n0 < g.N; n0 += nbmax) {
    const int nb = std::min(nbmax, g.N - n0);
    route(p, g, routed, gsrc, idx, D, n0, nb, st);
    GemmArgs a = gemm_args();             // dF[m][ci] = sum_pixel D[m][pixel] X[ci][pixel]
    a.M = M; a.N = g.Cin; a.K = Pi; a.transB = 1; a.lda = Pi; a.ldb = Pi; a.ldc = g.Cin;
    a.batch = nb; a.splitk = sk; a.strideA = (size_t)M * Pi; a.strideB = (size_t)g.Cin * Pi; a.strideC = nF;
    launch_gemm(a, D, x + (size_t)n0 * g.Cin * Pi, part, st);
    hipLaunchKernelGGL(k_gs_sum_acc, dim3((unsigned)((nF + 255) / 256)), dim3(256), 0, st, part, dF, nF, nb * sk,
                       n0 == 0 ? 1 : 0);
  }
  const int total = p->B * g.Cout * g.Cin;
  hipLaunchKernelGGL(k_gs_reduce_w, dim3((total + 255) / 256), dim3(256), 0, st, dF, dw, p->dev.fqt_ptr, p->dev.fqt_col,
                     p->dev.fqt_coef, p->B, g.Cout, g.Cin, g.kk);
}

}  // namespace

// Worth it from about a megaflop of products per call (measured: 16 x 16 maps with 8 -> 8 channels and 5 x 5 filters
// already break even); below that the single generic kernel wins on launches.
// Plan option gs = -1 / 1 switches the family off / on for every shape it can run.
bool gs_wanted(const rotconv_plan* p) {
  if (p->d.pool_op == ROTCONV_POOL_AVG) return false;
  if ((double)p->host.Q * p->d.Cout * p->kk * p->d.H * p->d.W * 4.0 > 3.0e9) return false;   // one image's products
  if (p->opt.gs) return p->opt.gs > 0;
  const double flops = 2.0 * p->d.N * p->d.H * p->d.W * p->d.Cin * p->d.Cout * p->kk * p->host.Q;
  return flops >= 1.0e6;
}

// The budget for the products of the images held at once (plan option gs_chunk_mb).
size_t gs_chunk_budget(const rotconv_plan* p) {
  if (p->opt.gs_chunk_mb > 0) return (size_t)p->opt.gs_chunk_mb << 20;
  if (p->opt.gs_chunk_mb < 0) return 0;       // one image at a time
  return (size_t)512 << 20;
}

size_t gs_ws_bytes(const rotconv_plan* p) { return gs_layout(p).total; }

void launch_gs_fwd(const rotconv_plan* p, const float* x, const float* w, float* y, void* ws, hipStream_t st) {
  forward(p, false, x, w, y, nullptr, ws, st);
}
void launch_gs_pool_fwd(const rotconv_plan* p, const float* x, const float* w, float* ypool, uint8_t* idx, void* ws,
                        hipStream_t st) {
  forward(p, true, x, w, ypool, idx, ws, st);
}
void launch_gs_bwd_data(const rotconv_plan* p, const float* dy, const float* w, float* dx, void* ws, hipStream_t st) {
  backward_data(p, false, dy, nullptr, w, dx, ws, st);
}
void launch_gs_pool_bwd_data(const rotconv_plan* p, const float* gpool, const uint8_t* idx, const float* w, float* dx,
                             void* ws, hipStream_t st) {
  backward_data(p, true, gpool, idx, w, dx, ws, st);
}
void launch_gs_bwd_weight(const rotconv_plan* p, const float* x, const float* dy, float* dw, void* ws, hipStream_t st) {
  backward_weight(p, false, x, dy, nullptr, dw, ws, st);
}
void launch_gs_pool_bwd_weight(const rotconv_plan* p, const float* x, const float* gpool, const uint8_t* idx, float* dw,
                               void* ws, hipStream_t st) {
  backward_weight(p, true, x, gpool, idx, dw, ws, st);
}

}  // namespace rotconv
