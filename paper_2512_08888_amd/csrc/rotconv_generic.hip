// Generic kernel family: correct for every descriptor the plan accepts (any k,
// stride, pad, R, angle set, mode).  Direct VALU convolution against the R
// rotated banks materialised once per call in scratch memory by a tiny
// expansion kernel.  The fast MFMA family covers the benchmark shapes; this one
// is the fallback and the path for tiny / odd shapes.
#include <hip/hip_runtime.h>

#include "rotconv_bf16.h"
#include "rotconv_kernels.h"

namespace rotconv {

Geom make_geom(const rotconv_plan* p) {
  Geom g;
  g.N = p->d.N; g.Cin = p->d.Cin; g.H = p->d.H; g.W = p->d.W; g.Cout = p->d.Cout; g.k = p->d.k; g.kk = p->kk;
  g.R = p->d.R; g.stride = p->d.stride; g.pad = p->d.pad; g.Ho = p->Ho; g.Wo = p->Wo; g.G = p->G; g.ng = p->ng;
  g.B = p->B; g.Q = p->host.Q;
  g.relu = 0;
  return g;
}

namespace {

constexpr int RT = 4;   // orientations per register chunk
constexpr int TT = 9;   // taps per register chunk in the weight gradient
constexpr int kBwdwTile = 16;

// Eq. 5 / Sec. III-D / Eq. 17: W^(r)[co,ci,t] = sum_e coef[r,t,e] * w[src[r,t,e]] (src = b*kk + u).
__global__ __launch_bounds__(256) void k_expand_bank(const float* __restrict__ w, float* __restrict__ wexp,
                                                     const int32_t* __restrict__ src, const float* __restrict__ coef,
                                                     const double* __restrict__ coef64, int R, int slices, int kk,
                                                     int round16) {
  const int total = R * slices * kk;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int t = e % kk;
  const int sl = (e / kk) % slices;
  const int r = e / (kk * slices);
  if (round16) {      // bf16 plans: the combination in fp64, rounded to fp32 and to bf16 once each
    double a64 = 0.0;
    for (int z = 0; z < kMaxNnz; ++z) {
      const int s = src[(r * kk + t) * kMaxNnz + z];
      if (s >= 0) a64 += coef64[(r * kk + t) * kMaxNnz + z] * (double)w[((s / kk) * slices + sl) * kk + s % kk];
    }
    wexp[e] = bf16_to_f32(f32_to_bf16((float)a64));
    return;
  }
  float acc = 0.f;
#pragma unroll
  for (int z = 0; z < kMaxNnz; ++z) {
    const int s = src[(r * kk + t) * kMaxNnz + z];
    if (s >= 0) {
      const int b = s / kk, u = s % kk;
      acc += coef[(r * kk + t) * kMaxNnz + z] * w[(b * slices + sl) * kk + u];
    }
  }
  wexp[e] = acc;
}

// Eq. 7 (and Eq. 10 when FUSED).  One thread = one output pixel of one filter
// (FUSED: of one pool group); orientations are processed RT at a time so the
// input value is loaded once per RT multiply-adds.  Weights are block-uniform.
template <bool FUSED>
__global__ __launch_bounds__(256) void k_fwd_generic(const float* __restrict__ x, const float* __restrict__ wexp,
                                                     float* __restrict__ yout, uint8_t* __restrict__ idx, Geom g) {
  const int P = g.Ho * g.Wo;
  const int p = blockIdx.x * 256 + threadIdx.x;
  const bool live = p < P;
  const int oy = live ? p / g.Wo : 0, ox = live ? p % g.Wo : 0;
  const int n = blockIdx.z;
  const int chan = blockIdx.y;                  // FUSED: co*ng + grp, else co
  const int co = FUSED ? chan / g.ng : chan;
  const int grp = FUSED ? chan % g.ng : 0;
  const int members = FUSED ? g.G : g.R;        // orientations handled by this block
  const int rstep = FUSED ? g.ng : 1;           // r = grp + j*rstep
  const float* xn = x + (size_t)n * g.Cin * g.H * g.W;
  const int wslice = g.Cin * g.kk;              // floats per (r, co)
  float best = 0.f;
  int best_r = grp;
  for (int j0 = 0; j0 < members; j0 += RT) {
    float acc[RT];
    const float* wr[RT];
#pragma unroll
    for (int rr = 0; rr < RT; ++rr) {
      acc[rr] = 0.f;
      const int j = (j0 + rr < members) ? j0 + rr : j0;  // clamp: duplicates are discarded below
      const int r = grp + j * rstep;
      wr[rr] = wexp + ((size_t)r * g.Cout + co) * wslice;
    }
    for (int ci = 0; ci < g.Cin; ++ci)
      for (int i = 0; i < g.k; ++i) {
        const int h = oy * g.stride + i - g.pad;
        const bool hin = live && h >= 0 && h < g.H;
        for (int jx = 0; jx < g.k; ++jx) {
          const int w = ox * g.stride + jx - g.pad;
          const float xv = (hin && w >= 0 && w < g.W) ? xn[((size_t)ci * g.H + h) * g.W + w] : 0.f;
          const int t = (ci * g.k + i) * g.k + jx;
#pragma unroll
          for (int rr = 0; rr < RT; ++rr) acc[rr] += wr[rr][t] * xv;
        }
      }
#pragma unroll
    for (int rr = 0; rr < RT; ++rr) {
      if (j0 + rr >= members) continue;
      const int r = grp + (j0 + rr) * rstep;
      if (FUSED) {
        if ((j0 + rr) == 0 || acc[rr] > best) { best = acc[rr]; best_r = r; }
      } else if (live) {
        yout[(((size_t)n * g.Cout + co) * g.R + r) * P + p] = acc[rr];
      }
    }
  }
  if (FUSED && live) {
    const size_t q = ((size_t)n * g.Cout * g.ng + chan) * P + p;
    const bool dead = g.relu && !(best > 0.f);        // fused ReLU: nothing flows back through this element
    yout[q] = dead ? 0.f : best;
    idx[q] = dead ? (uint8_t)255 : (uint8_t)best_r;
  }
}

// Eq. 10 on a materialised y.
// T = float, or uint16_t holding bfloat16 (compared as fp32; the winner's bits are copied unchanged)
template <typename T> __device__ __forceinline__ float as_f32(T v);
template <> __device__ __forceinline__ float as_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float as_f32<uint16_t>(uint16_t v) { return bf16_to_f32(v); }

template <typename T>
__global__ __launch_bounds__(256) void k_maxpool_fwd(const T* __restrict__ y, T* __restrict__ ypool,
                                                     uint8_t* __restrict__ idx, Geom g) {
  const int P = g.Ho * g.Wo;
  const int p = blockIdx.x * 256 + threadIdx.x;
  if (p >= P) return;
  const int chan = blockIdx.y, n = blockIdx.z;
  const int co = chan / g.ng, grp = chan % g.ng;
  const T* yb = y + ((size_t)n * g.Cout + co) * g.R * P + p;
  T best_raw = yb[(size_t)grp * P];
  float best = as_f32<T>(best_raw);
  int best_r = grp;
  for (int r = grp + g.ng; r < g.R; r += g.ng) {
    const T raw = yb[(size_t)r * P];
    const float v = as_f32<T>(raw);
    if (v > best) { best = v; best_raw = raw; best_r = r; }
  }
  const size_t q = ((size_t)n * g.Cout * g.ng + chan) * P + p;
  const bool dead = g.relu && !(best > 0.f);
  ypool[q] = dead ? T(0) : best_raw;
  idx[q] = dead ? (uint8_t)255 : (uint8_t)best_r;
}

// Eq. 12.
template <typename T>
__global__ __launch_bounds__(256) void k_maxpool_bwd(const T* __restrict__ gpool, const uint8_t* __restrict__ idx,
                                                     T* __restrict__ dy, Geom g) {
  const int P = g.Ho * g.Wo;
  const int p = blockIdx.x * 256 + threadIdx.x;
  if (p >= P) return;
  const int chan = blockIdx.y, n = blockIdx.z;   // chan = co*R + r
  const int co = chan / g.R, r = chan % g.R;
  const size_t q = (((size_t)n * g.Cout + co) * g.ng + r % g.ng) * P + p;
  dy[((size_t)n * g.Cout * g.R + chan) * P + p] = (idx[q] == r) ? gpool[q] : T(0);
}

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ uint16_t from_f32<uint16_t>(float v) { return f32_to_bf16(v); }

// Eq. 9: mean over each pool group (T = float, or uint16_t holding bfloat16: summed in fp32, rounded once).
template <typename T>
__global__ __launch_bounds__(256) void k_avgpool_fwd(const T* __restrict__ y, T* __restrict__ ypool, Geom g) {
  const int P = g.Ho * g.Wo;
  const int p = blockIdx.x * 256 + threadIdx.x;
  if (p >= P) return;
  const int chan = blockIdx.y, n = blockIdx.z;
  const int co = chan / g.ng, grp = chan % g.ng;
  const T* yb = y + ((size_t)n * g.Cout + co) * g.R * P + p;
  float s = 0.f;
  for (int r = grp; r < g.R; r += g.ng) s += as_f32<T>(yb[(size_t)r * P]);
  ypool[((size_t)n * g.Cout * g.ng + chan) * P + p] = from_f32<T>(s * (1.0f / (float)g.G));
}

// Eq. 11: every member of the group receives gpool / G.
template <typename T>
__global__ __launch_bounds__(256) void k_avgpool_bwd(const T* __restrict__ gpool, T* __restrict__ dy, Geom g) {
  const int P = g.Ho * g.Wo;
  const int p = blockIdx.x * 256 + threadIdx.x;
  if (p >= P) return;
  const int chan = blockIdx.y, n = blockIdx.z;   // chan = co*R + r
  const int co = chan / g.R, r = chan % g.R;
  const size_t q = (((size_t)n * g.Cout + co) * g.ng + r % g.ng) * P + p;
  dy[((size_t)n * g.Cout * g.R + chan) * P + p] = from_f32<T>(as_f32<T>(gpool[q]) * (1.0f / (float)g.G));
}

// Group-averaged bank: wavg[(co*ng+grp)][ci][t] = (1/G) sum_{r mod ng == grp} wexp[r][co][ci][t].
__global__ __launch_bounds__(256) void k_avg_bank(const float* __restrict__ wexp, float* __restrict__ wavg, int R,
                                                  int ng, int Cout, int per /* Cin*kk */) {
  const int total = Cout * ng * per;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int t = e % per, chan = e / per;
  const int co = chan / ng, grp = chan % ng;
  float s = 0.f;
  for (int r = grp; r < R; r += ng) s += wexp[((size_t)r * Cout + co) * per + t];
  wavg[e] = s * (1.0f / (float)(R / ng));
}
// Adjoint of k_avg_bank: rep[r][co][ci][t] = dwavg[(co*ng + r mod ng)][ci][t] / G.
__global__ __launch_bounds__(256) void k_avg_bank_bwd(const float* __restrict__ dwavg, float* __restrict__ rep, int R,
                                                      int ng, int Cout, int per) {
  const int total = R * Cout * per;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int t = e % per, co = (e / per) % Cout, r = e / (per * Cout);
  rep[e] = dwavg[((size_t)co * ng + r % ng) * per + t] * (1.0f / (float)(R / ng));
}
__global__ __launch_bounds__(256) void k_fill_u8(uint8_t* __restrict__ p, size_t n, uint8_t v) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = v;
}

// Eq. 13 + 15 (with Eq. 12 folded in when FUSED: only the winning orientation of
// each pooled element contributes, so the loop runs over pooled channels and the
// weight is looked up by the stored orientation index).
template <bool FUSED>
__global__ __launch_bounds__(256) void k_bwd_data_generic(const float* __restrict__ gin, const uint8_t* __restrict__ idx,
                                                          const float* __restrict__ wexp, float* __restrict__ dx,
                                                          Geom g) {
  const int HW = g.H * g.W, P = g.Ho * g.Wo;
  const int pix = blockIdx.x * 256 + threadIdx.x;
  if (pix >= HW) return;
  const int h = pix / g.W, w = pix % g.W;
  const int ci = blockIdx.y, n = blockIdx.z;
  float acc = 0.f;
  for (int i = 0; i < g.k; ++i) {
    const int ty = h + g.pad - i;
    if (ty < 0 || ty % g.stride) continue;
    const int oy = ty / g.stride;
    if (oy >= g.Ho) continue;
    for (int j = 0; j < g.k; ++j) {
      const int tx = w + g.pad - j;
      if (tx < 0 || tx % g.stride) continue;
      const int ox = tx / g.stride;
      if (ox >= g.Wo) continue;
      const int t = i * g.k + j;
      const int po = oy * g.Wo + ox;
      if (FUSED) {
        const int Cp = g.Cout * g.ng;
        for (int c = 0; c < Cp; ++c) {
          const size_t q = ((size_t)n * Cp + c) * P + po;
          const int r = idx[q];
          if (r < g.R && r % g.ng == c % g.ng)
            acc += wexp[(((size_t)r * g.Cout + c / g.ng) * g.Cin + ci) * g.kk + t] * gin[q];
        }
      } else {
        for (int co = 0; co < g.Cout; ++co)
          for (int r = 0; r < g.R; ++r)
            acc += wexp[(((size_t)r * g.Cout + co) * g.Cin + ci) * g.kk + t] *
                   gin[(((size_t)n * g.Cout + co) * g.R + r) * P + po];
      }
    }
  }
  dx[((size_t)n * g.Cin + ci) * HW + pix] = acc;
}

// Eq. 14 (with Eq. 12 folded in when FUSED).  Block = 16 ci x 16 co; every thread
// owns one (co,ci) pair and keeps RT x TT partial sums in registers while the
// block walks a contiguous range of output pixels; ranges ("splits") are summed
// afterwards in a fixed order, so the result does not depend on scheduling.
template <bool FUSED>
__global__ __launch_bounds__(256) void k_bwd_weight_generic(const float* __restrict__ x, const float* __restrict__ gin,
                                                            const uint8_t* __restrict__ idx,
                                                            float* __restrict__ partial, Geom g, int splits) {
  const int P = g.Ho * g.Wo;
  const int total = g.N * P;
  const int ci = blockIdx.x * kBwdwTile + (threadIdx.x % kBwdwTile);
  const int co = blockIdx.y * kBwdwTile + (threadIdx.x / kBwdwTile);
  const int split = blockIdx.z;
  const int chunk = (total + splits - 1) / splits;
  const int p_begin = split * chunk;
  const int p_end = min(total, p_begin + chunk);
  const bool live = ci < g.Cin && co < g.Cout;
  const int cis = live ? ci : 0, cos = live ? co : 0;
  const size_t wexp_n = (size_t)g.R * g.Cout * g.Cin * g.kk;
  float* out = partial + (size_t)split * wexp_n;
  for (int r0 = 0; r0 < g.R; r0 += RT)
    for (int t0 = 0; t0 < g.kk; t0 += TT) {
      float acc[RT][TT];
      int di[TT], dj[TT];
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) {
        const int t = min(t0 + tt, g.kk - 1);
        di[tt] = t / g.k - g.pad;
        dj[tt] = t % g.k - g.pad;
#pragma unroll
        for (int rr = 0; rr < RT; ++rr) acc[rr][tt] = 0.f;
      }
      for (int pi = p_begin; pi < p_end; ++pi) {
        const int n = pi / P, po = pi % P;
        const int oy = po / g.Wo, ox = po % g.Wo;
        float m[RT];
#pragma unroll
        for (int rr = 0; rr < RT; ++rr) {
          const int r = min(r0 + rr, g.R - 1);
          if (FUSED) {
            const size_t q = (((size_t)n * g.Cout + cos) * g.ng + r % g.ng) * P + po;
            m[rr] = (idx[q] == r) ? gin[q] : 0.f;
          } else {
            m[rr] = gin[(((size_t)n * g.Cout + cos) * g.R + r) * P + po];
          }
        }
        const float* xc = x + ((size_t)n * g.Cin + cis) * g.H * g.W;
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
          const int h = oy * g.stride + di[tt], w = ox * g.stride + dj[tt];
          const float xv = (h >= 0 && h < g.H && w >= 0 && w < g.W) ? xc[h * g.W + w] : 0.f;
#pragma unroll
          for (int rr = 0; rr < RT; ++rr) acc[rr][tt] += m[rr] * xv;
        }
      }
      if (live) {
#pragma unroll
        for (int rr = 0; rr < RT; ++rr)
#pragma unroll
          for (int tt = 0; tt < TT; ++tt)
            if (r0 + rr < g.R && t0 + tt < g.kk)
              out[(((size_t)(r0 + rr) * g.Cout + co) * g.Cin + ci) * g.kk + t0 + tt] = acc[rr][tt];
      }
    }
}

// Eq. 16 generalised: sum the splits in order, then apply the transposed expansion.
// One thread per base element dw[b][co][ci][u].
__global__ __launch_bounds__(256) void k_reduce_bank(const float* __restrict__ partial, float* __restrict__ dw,
                                                     const int32_t* __restrict__ tr_ptr,
                                                     const int32_t* __restrict__ tr_col,
                                                     const float* __restrict__ tr_coef, int B, int slices, int kk,
                                                     int splits, size_t bank_n) {
  const int total = B * slices * kk;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int u = e % kk;
  const int sl = (e / kk) % slices;
  const int b = e / (kk * slices);
  float acc = 0.f;
  for (int z = tr_ptr[b * kk + u]; z < tr_ptr[b * kk + u + 1]; ++z) {
    const int col = tr_col[z];  // r*kk + t  (or q*kk + t)
    const int r = col / kk, t = col % kk;
    float s = 0.f;
    for (int sp = 0; sp < splits; ++sp) s += partial[(size_t)sp * bank_n + ((size_t)r * slices + sl) * kk + t];
    acc += tr_coef[z] * s;
  }
  dw[e] = acc;
}

}  // namespace

int generic_bwdw_splits(const rotconv_plan* p) {
  const long tiles = (long)((p->d.Cin + kBwdwTile - 1) / kBwdwTile) * ((p->d.Cout + kBwdwTile - 1) / kBwdwTile);
  const long total = (long)p->d.N * p->Ho * p->Wo;
  const double bank_bytes = 4.0 * p->d.R * p->d.Cout * p->d.Cin * p->kk;
  long s = (2048 + tiles - 1) / tiles;
  s = std::min(s, std::max(1L, total / 64));
  s = std::min(s, std::max(1L, (long)(268435456.0 / bank_bytes)));
  s = std::min(s, 65535L);
  return (int)std::max(1L, s);
}

size_t generic_ws_bytes(const rotconv_plan* p) {
  const size_t bank = (size_t)p->d.R * p->d.Cout * p->d.Cin * p->kk * sizeof(float);
  const size_t a = (bank + 255) / 256 * 256;
  return std::max(a, (size_t)generic_bwdw_splits(p) * bank);
}

void launch_expand_bank(const rotconv_plan* p, const float* w, float* wexp, hipStream_t st) {
  const int slices = p->d.Cout * p->d.Cin;
  const int total = p->d.R * slices * p->kk;
  hipLaunchKernelGGL(k_expand_bank, dim3((total + 255) / 256), dim3(256), 0, st, w, wexp, p->dev.exp_src,
                     p->dev.exp_coef, p->dev.exp_coef64, p->d.R, slices, p->kk, p->d.dtype == ROTCONV_BF16 ? 1 : 0);
}

void launch_fwd_generic(const rotconv_plan* p, const float* x, const float* wexp, float* y, hipStream_t st) {
  const Geom g = make_geom(p);
  dim3 grid((g.Ho * g.Wo + 255) / 256, g.Cout, g.N);
  hipLaunchKernelGGL(k_fwd_generic<false>, grid, dim3(256), 0, st, x, wexp, y, (uint8_t*)nullptr, g);
}

void launch_pool_fwd_generic(const rotconv_plan* p, const float* x, const float* wexp, float* ypool, uint8_t* idx,
                             hipStream_t st) {
  Geom g = make_geom(p);
  g.relu = p->d.activation == ROTCONV_ACT_RELU;
  dim3 grid((g.Ho * g.Wo + 255) / 256, g.Cout * g.ng, g.N);
  hipLaunchKernelGGL(k_fwd_generic<true>, grid, dim3(256), 0, st, x, wexp, ypool, idx, g);
}

void launch_maxpool_fwd(const rotconv_plan* p, const float* y, float* ypool, uint8_t* idx, hipStream_t st, bool relu) {
  Geom g = make_geom(p);
  g.relu = relu && p->d.activation == ROTCONV_ACT_RELU;
  dim3 grid((g.Ho * g.Wo + 255) / 256, g.Cout * g.ng, g.N);
  hipLaunchKernelGGL(k_maxpool_fwd<float>, grid, dim3(256), 0, st, y, ypool, idx, g);
}

void launch_avgpool_fwd(const rotconv_plan* p, const float* y, float* ypool, hipStream_t st) {
  const Geom g = make_geom(p);
  dim3 grid((g.Ho * g.Wo + 255) / 256, g.Cout * g.ng, g.N);
  hipLaunchKernelGGL(k_avgpool_fwd<float>, grid, dim3(256), 0, st, y, ypool, g);
}
void launch_avgpool_fwd_bf16(const rotconv_plan* p, const uint16_t* y, uint16_t* ypool, hipStream_t st) {
  const Geom g = make_geom(p);
  dim3 grid((g.Ho * g.Wo + 255) / 256, g.Cout * g.ng, g.N);
  hipLaunchKernelGGL(k_avgpool_fwd<uint16_t>, grid, dim3(256), 0, st, y, ypool, g);
}
void launch_avgpool_bwd_bf16(const rotconv_plan* p, const uint16_t* gpool, uint16_t* dy, hipStream_t st) {
  const Geom g = make_geom(p);
  dim3 grid((g.Ho * g.Wo + 255) / 256, g.Cout * g.R, g.N);
  hipLaunchKernelGGL(k_avgpool_bwd<uint16_t>, grid, dim3(256), 0, st, gpool, dy, g);
}
void launch_avgpool_bwd(const rotconv_plan* p, const float* gpool, float* dy, hipStream_t st) {
  const Geom g = make_geom(p);
  dim3 grid((g.Ho * g.Wo + 255) / 256, g.Cout * g.R, g.N);
  hipLaunchKernelGGL(k_avgpool_bwd<float>, grid, dim3(256), 0, st, gpool, dy, g);
}
void launch_avg_bank(const rotconv_plan* p, const float* wexp, float* wavg, hipStream_t st) {
  const int per = p->d.Cin * p->kk, total = p->d.Cout * p->ng * per;
  hipLaunchKernelGGL(k_avg_bank, dim3((total + 255) / 256), dim3(256), 0, st, wexp, wavg, p->d.R, p->ng, p->d.Cout, per);
}
void launch_avg_bank_bwd(const rotconv_plan* p, const float* dwavg, float* rep, float* dw, hipStream_t st) {
  const int per = p->d.Cin * p->kk, total = p->d.R * p->d.Cout * per;
  hipLaunchKernelGGL(k_avg_bank_bwd, dim3((total + 255) / 256), dim3(256), 0, st, dwavg, rep, p->d.R, p->ng, p->d.Cout,
                     per);
  const int slices = p->d.Cout * p->d.Cin, tot = p->B * slices * p->kk;
  hipLaunchKernelGGL(k_reduce_bank, dim3((tot + 255) / 256), dim3(256), 0, st, rep, dw, p->dev.tr_ptr, p->dev.tr_col,
                     p->dev.tr_coef, p->B, slices, p->kk, 1, (size_t)p->d.R * slices * p->kk);
}
void launch_fill_u8(uint8_t* p, size_t n, uint8_t v, hipStream_t st) {
  const unsigned blocks = (unsigned)std::max<size_t>(1, std::min<size_t>((n + 255) / 256, 4096));
  hipLaunchKernelGGL(k_fill_u8, dim3(blocks), dim3(256), 0, st, p, n, v);
}

void launch_maxpool_fwd_bf16(const rotconv_plan* p, const uint16_t* y, uint16_t* ypool, uint8_t* idx, hipStream_t st) {
  const Geom g = make_geom(p);
  dim3 grid((g.Ho * g.Wo + 255) / 256, g.Cout * g.ng, g.N);
  hipLaunchKernelGGL(k_maxpool_fwd<uint16_t>, grid, dim3(256), 0, st, y, ypool, idx, g);
}

void launch_maxpool_bwd(const rotconv_plan* p, const float* gpool, const uint8_t* idx, float* dy, hipStream_t st) {
  const Geom g = make_geom(p);
  dim3 grid((g.Ho * g.Wo + 255) / 256, g.Cout * g.R, g.N);
  hipLaunchKernelGGL(k_maxpool_bwd<float>, grid, dim3(256), 0, st, gpool, idx, dy, g);
}

void launch_maxpool_bwd_bf16(const rotconv_plan* p, const uint16_t* gpool, const uint8_t* idx, uint16_t* dy,
                             hipStream_t st) {
  const Geom g = make_geom(p);
  dim3 grid((g.Ho * g.Wo + 255) / 256, g.Cout * g.R, g.N);
  hipLaunchKernelGGL(k_maxpool_bwd<uint16_t>, grid, dim3(256), 0, st, gpool, idx, dy, g);
}

void launch_bwd_data_generic(const rotconv_plan* p, const float* dy, const float* wexp, float* dx, hipStream_t st) {
  const Geom g = make_geom(p);
  dim3 grid((g.H * g.W + 255) / 256, g.Cin, g.N);
  hipLaunchKernelGGL(k_bwd_data_generic<false>, grid, dim3(256), 0, st, dy, (const uint8_t*)nullptr, wexp, dx, g);
}

void launch_pool_bwd_data_generic(const rotconv_plan* p, const float* gpool, const uint8_t* idx, const float* wexp,
                                  float* dx, hipStream_t st) {
  const Geom g = make_geom(p);
  dim3 grid((g.H * g.W + 255) / 256, g.Cin, g.N);
  hipLaunchKernelGGL(k_bwd_data_generic<true>, grid, dim3(256), 0, st, gpool, idx, wexp, dx, g);
}

void launch_bwd_weight_generic(const rotconv_plan* p, const float* x, const float* dy, const float* gpool,
                               const uint8_t* idx, float* partial, float* dw, hipStream_t st) {
  const Geom g = make_geom(p);
  const int splits = p->bwdw_splits;
  dim3 grid((g.Cin + kBwdwTile - 1) / kBwdwTile, (g.Cout + kBwdwTile - 1) / kBwdwTile, splits);
  if (dy)
    hipLaunchKernelGGL(k_bwd_weight_generic<false>, grid, dim3(256), 0, st, x, dy, (const uint8_t*)nullptr, partial, g,
                       splits);
  else
    hipLaunchKernelGGL(k_bwd_weight_generic<true>, grid, dim3(256), 0, st, x, gpool, idx, partial, g, splits);
  const int slices = g.Cout * g.Cin;
  const int total = g.B * slices * g.kk;
  const size_t bank_n = (size_t)g.R * slices * g.kk;
  hipLaunchKernelGGL(k_reduce_bank, dim3((total + 255) / 256), dim3(256), 0, st, partial, dw, p->dev.tr_ptr,
                     p->dev.tr_col, p->dev.tr_coef, g.B, slices, g.kk, splits, bank_n);
}

}  // namespace rotconv
