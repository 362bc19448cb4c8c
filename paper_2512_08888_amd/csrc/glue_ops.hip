// Network glue around the rotation convolution (see include/unetglue.h): streaming
// elementwise / window kernels (HBM-bound) and the GEMM-shaped layers mapped onto the
// matrix-core GEMM of glue_gemm.hip.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "glue_internal.h"
#include "rotconv.h"
#include "rotconv_bf16.h"
#include "unetglue.h"

namespace rotconv {
namespace {

int finish() { return hipGetLastError() == hipSuccess ? ROTCONV_OK : ROTCONV_ERR_LAUNCH; }
unsigned blocks_for(size_t n) { return (unsigned)std::max<size_t>(1, std::min<size_t>((n + 255) / 256, 1u << 20)); }

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Element access for the two storage types: fp32, and bfloat16 kept in uint16_t (arithmetic is fp32 in
// both cases; a bf16 result is rounded once, to nearest even).  V = elements of one 16-byte access.
template <typename T> struct Elt;
template <> struct Elt<float> {
  static constexpr int V = 4;
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
  static __device__ __forceinline__ void ldv(const float* p, float* v) {
    const f4 a = *reinterpret_cast<const f4*>(p);
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = a[k];
  }
  static __device__ __forceinline__ void stv(float* p, const float* v) {
    *reinterpret_cast<f4*>(p) = f4{v[0], v[1], v[2], v[3]};
  }
  static __device__ __forceinline__ void ldh(const float* p, float* v) {   // half a vector: 8 bytes
    const float2 a = *reinterpret_cast<const float2*>(p);
    v[0] = a.x; v[1] = a.y;
  }
  static __device__ __forceinline__ void sth(float* p, const float* v) {
    *reinterpret_cast<float2*>(p) = make_float2(v[0], v[1]);
  }
};
template <> struct Elt<uint16_t> {
  static constexpr int V = 8;
  static __device__ __forceinline__ float ld(const uint16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void st(uint16_t* p, float v) { *p = f32_to_bf16(v); }
  static __device__ __forceinline__ void ldv(const uint16_t* p, float* v) {
    const u4 a = *reinterpret_cast<const u4*>(p);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      v[2 * k] = __uint_as_float(a[k] << 16);
      v[2 * k + 1] = __uint_as_float(a[k] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void stv(uint16_t* p, const float* v) {
    u4 a;
#pragma unroll
    for (int k = 0; k < 4; ++k) a[k] = (uint32_t)f32_to_bf16(v[2 * k]) | ((uint32_t)f32_to_bf16(v[2 * k + 1]) << 16);
    *reinterpret_cast<u4*>(p) = a;
  }
  static __device__ __forceinline__ void ldh(const uint16_t* p, float* v) {
    const uint2 a = *reinterpret_cast<const uint2*>(p);
    v[0] = __uint_as_float(a.x << 16); v[1] = __uint_as_float(a.x & 0xffff0000u);
    v[2] = __uint_as_float(a.y << 16); v[3] = __uint_as_float(a.y & 0xffff0000u);
  }
  static __device__ __forceinline__ void sth(uint16_t* p, const float* v) {
    *reinterpret_cast<uint2*>(p) = make_uint2((uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16),
                                              (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16));
  }
};

// Streaming kernels: one 16-byte access per lane when the shapes and pointers allow (VEC), else one element.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void k_relu_fwd(const T* __restrict__ x, T* __restrict__ y, size_t n) {
  constexpr int V = VEC ? Elt<T>::V : 1;
  const size_t nv = n / V;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nv; i += (size_t)gridDim.x * 256) {
    if (VEC) {
      float v[Elt<T>::V];
      Elt<T>::ldv(x + i * V, v);
#pragma unroll
      for (int k = 0; k < V; ++k) v[k] = fmaxf(v[k], 0.f);
      Elt<T>::stv(y + i * V, v);
    } else {
      Elt<T>::st(y + i, fmaxf(Elt<T>::ld(x + i), 0.f));
    }
  }
  const size_t t = nv * V + (size_t)blockIdx.x * 256 + threadIdx.x;    // the last n % V elements
  if (VEC && t < n) Elt<T>::st(y + t, fmaxf(Elt<T>::ld(x + t), 0.f));
}
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void k_relu_bwd(const T* __restrict__ y, const T* __restrict__ dy,
                                                  T* __restrict__ dx, size_t n) {
  constexpr int V = VEC ? Elt<T>::V : 1;
  const size_t nv = n / V;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nv; i += (size_t)gridDim.x * 256) {
    if (VEC) {
      float a[Elt<T>::V], d[Elt<T>::V];
      Elt<T>::ldv(y + i * V, a);
      Elt<T>::ldv(dy + i * V, d);
#pragma unroll
      for (int k = 0; k < V; ++k) d[k] = a[k] > 0.f ? d[k] : 0.f;
      Elt<T>::stv(dx + i * V, d);
    } else {
      Elt<T>::st(dx + i, Elt<T>::ld(y + i) > 0.f ? Elt<T>::ld(dy + i) : 0.f);
    }
  }
  const size_t t = nv * V + (size_t)blockIdx.x * 256 + threadIdx.x;
  if (VEC && t < n) Elt<T>::st(dx + t, Elt<T>::ld(y + t) > 0.f ? Elt<T>::ld(dy + t) : 0.f);
}

// VEC: one thread per 16 bytes of an input row pair (V columns = V/2 windows); else one thread per window.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void k_maxpool2_fwd(const T* __restrict__ x, T* __restrict__ y,
                                                      uint8_t* __restrict__ idx, size_t planes, int H, int W) {
  constexpr int NW = VEC ? Elt<T>::V / 2 : 1;   // windows per thread
  const int Ho = H / 2, Wo = W / 2, Wv = Wo / NW;
  const size_t total = planes * Ho * Wv;
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const int ox = (int)(e % Wv) * NW, oy = (int)((e / Wv) % Ho);
    const size_t pl = e / ((size_t)Wv * Ho);
    const T* p = x + (pl * H + 2 * oy) * W + 2 * ox;
    float r0[2 * NW], r1[2 * NW];
    if (VEC) {
      Elt<T>::ldv(p, r0);
      Elt<T>::ldv(p + W, r1);
    } else {
      r0[0] = Elt<T>::ld(p); r0[1] = Elt<T>::ld(p + 1); r1[0] = Elt<T>::ld(p + W); r1[1] = Elt<T>::ld(p + W + 1);
    }
    float best[NW];
    uint32_t packed = 0;
#pragma unroll
    for (int k = 0; k < NW; ++k) {
      int bi = 0;
      best[k] = r0[2 * k];
      if (r0[2 * k + 1] > best[k]) { best[k] = r0[2 * k + 1]; bi = 1; }
      if (r1[2 * k] > best[k]) { best[k] = r1[2 * k]; bi = 2; }
      if (r1[2 * k + 1] > best[k]) { best[k] = r1[2 * k + 1]; bi = 3; }
      packed |= (uint32_t)bi << (8 * k);
    }
    const size_t o = (pl * Ho + oy) * Wo + ox;
    if (VEC) {
      Elt<T>::sth(y + o, best);
      if (NW == 2) *reinterpret_cast<uint16_t*>(idx + o) = (uint16_t)packed;
      else *reinterpret_cast<uint32_t*>(idx + o) = packed;
    } else {
      Elt<T>::st(y + o, best[0]);
      idx[o] = (uint8_t)packed;
    }
  }
}
// VEC: one thread per 16 bytes of an input row (V columns, V/2 windows); else one thread per input element.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void k_maxpool2_bwd(const T* __restrict__ dy, const uint8_t* __restrict__ idx,
                                                      T* __restrict__ dx, size_t planes, int H, int W, int acc) {
  constexpr int V = VEC ? Elt<T>::V : 1;
  const int Ho = H / 2, Wo = W / 2, Wv = W / V;
  const size_t total = planes * H * Wv;
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const int xx = (int)(e % Wv) * V, yy = (int)((e / Wv) % H);
    const size_t pl = e / ((size_t)Wv * H);
    const size_t o = (pl * Ho + yy / 2) * Wo + xx / 2;
    const size_t i = (pl * H + yy) * W + xx;
    if (VEC) {
      constexpr int NW = Elt<T>::V / 2;
      float d[NW], v[Elt<T>::V];
      Elt<T>::ldh(dy + o, d);
      const uint32_t w = NW == 2 ? (uint32_t)*reinterpret_cast<const uint16_t*>(idx + o)
                                 : *reinterpret_cast<const uint32_t*>(idx + o);
      const uint32_t r = 2 * (yy & 1);
#pragma unroll
      for (int k = 0; k < NW; ++k) {
        const uint32_t b = (w >> (8 * k)) & 0xff;
        v[2 * k] = b == r ? d[k] : 0.f;
        v[2 * k + 1] = b == r + 1 ? d[k] : 0.f;
      }
      if (acc) {
        float old[Elt<T>::V];
        Elt<T>::ldv(dx + i, old);
#pragma unroll
        for (int k = 0; k < V; ++k) v[k] += old[k];
      }
      Elt<T>::stv(dx + i, v);
    } else {
      const float v = idx[o] == (uint8_t)(2 * (yy & 1) + (xx & 1)) ? Elt<T>::ld(dy + o) : 0.f;
      Elt<T>::st(dx + i, acc ? Elt<T>::ld(dx + i) + v : v);
    }
  }
}

// na, nb: elements per image of the two parts.  VEC needs both divisible by V.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void k_concat2(const T* __restrict__ a, const T* __restrict__ b,
                                                 T* __restrict__ out, int N, size_t na, size_t nb) {
  constexpr int V = VEC ? Elt<T>::V : 1;
  const size_t va = na / V, vb = nb / V, total = (size_t)N * (va + vb);
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const size_t n = e / (va + vb), r = e % (va + vb);
    const T* src = r < va ? a + (n * va + r) * V : b + (n * vb + (r - va)) * V;
    if (VEC) *reinterpret_cast<u4*>(out + e * V) = *reinterpret_cast<const u4*>(src);
    else out[e] = *src;
  }
}
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void k_split2(const T* __restrict__ dcat, T* __restrict__ da,
                                                T* __restrict__ db, int N, size_t na, size_t nb, int acc) {
  constexpr int V = VEC ? Elt<T>::V : 1;
  const size_t va = na / V, vb = nb / V, total = (size_t)N * (va + vb);
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const size_t n = e / (va + vb), r = e % (va + vb);
    if (r >= va) {
      T* d = db + (n * vb + (r - va)) * V;
      if (VEC) *reinterpret_cast<u4*>(d) = *reinterpret_cast<const u4*>(dcat + e * V);
      else *d = dcat[e];
    } else if (!acc) {
      T* d = da + (n * va + r) * V;
      if (VEC) *reinterpret_cast<u4*>(d) = *reinterpret_cast<const u4*>(dcat + e * V);
      else *d = dcat[e];
    } else if (VEC) {
      float v[Elt<T>::V], old[Elt<T>::V];
      T* d = da + (n * va + r) * V;
      Elt<T>::ldv(dcat + e * V, v);
      Elt<T>::ldv(d, old);
#pragma unroll
      for (int k = 0; k < V; ++k) v[k] += old[k];
      Elt<T>::stv(d, v);
    } else {
      T* d = da + n * va + r;
      Elt<T>::st(d, Elt<T>::ld(d) + Elt<T>::ld(dcat + e));
    }
  }
}

// dlogits = (softmax - onehot) * inv; the workgroup's pixel losses, added in a fixed order (a thread's pixels in
// sequence, then a tree over the threads), go to part[blockIdx.x]
template <typename T>
__global__ __launch_bounds__(256) void k_softmax_ce(const T* __restrict__ logits, const int32_t* __restrict__ labels,
                                                    float* __restrict__ part, T* __restrict__ dl, int N, int K,
                                                    size_t P, float inv) {
  __shared__ float red[256];
  const size_t total = (size_t)N * P;
  float mine = 0.f;
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
    const size_t n = e / P, p = e % P;
    const T* lg = logits + n * K * P + p;
    float m = Elt<T>::ld(lg);
    for (int k = 1; k < K; ++k) m = fmaxf(m, Elt<T>::ld(lg + (size_t)k * P));
    float s = 0.f;
    for (int k = 0; k < K; ++k) s += expf(Elt<T>::ld(lg + (size_t)k * P) - m);
    const int lab = labels[e];
    const bool valid = lab >= 0 && lab < K;      // a label outside 0..K-1 contributes nothing
    const float lse = m + logf(s);
    mine += valid ? lse - Elt<T>::ld(lg + (size_t)(valid ? lab : 0) * P) : 0.f;
    T* d = dl + n * K * P + p;
    for (int k = 0; k < K; ++k)
      Elt<T>::st(d + (size_t)k * P,
                 valid ? (expf(Elt<T>::ld(lg + (size_t)k * P) - lse) - (k == lab ? 1.f : 0.f)) * inv : 0.f);
  }
  red[threadIdx.x] = mine;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) part[blockIdx.x] = red[0];
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

// ---- 1x1 head with few output channels (the class scores): streaming kernels on the vector ALU ----
// A 128-row matrix-core tile would be nine tenths padding for six classes; the layer is HBM-bound (it reads
// or writes the Cin-channel map once), so a lane owns one 16-byte vector of consecutive pixels and walks the
// channels.  w sits in LDS as fp32 [ci][HEAD_CO] (zero beyond Cout).  Sums run in a fixed order.
constexpr int HEAD_CO = 8;         // at most this many output channels
constexpr int HEAD_CIN = 1024;     // at most this many input channels (LDS copy of w)
constexpr int HEAD_PARTS = 256;    // workgroups (= partial sums) of the weight gradient, at most

template <typename T>
__device__ __forceinline__ void head_load_w(const T* __restrict__ w, float* wl, int Cin, int Cout) {
  for (int i = threadIdx.x; i < Cin * HEAD_CO; i += 256) {
    const int ci = i / HEAD_CO, co = i % HEAD_CO;
    wl[i] = co < Cout ? Elt<T>::ld(w + (size_t)co * Cin + ci) : 0.f;
  }
  __syncthreads();
}

// y[n][co][p] = sum_ci w[co][ci] x[n][ci][p]
template <typename T>
__global__ __launch_bounds__(256) void k_head_fwd(const T* __restrict__ x, const T* __restrict__ w, T* __restrict__ y,
                                                  int Cin, int Cout, size_t P, size_t nvec) {
  constexpr int V = Elt<T>::V;
  extern __shared__ float wl[];
  head_load_w(w, wl, Cin, Cout);
  const size_t pv = P / V;
  for (size_t v = (size_t)blockIdx.x * 256 + threadIdx.x; v < nvec; v += (size_t)gridDim.x * 256) {
    const size_t n = v / pv, p = (v - n * pv) * V;
    const T* xp = x + n * Cin * P + p;
    float acc[HEAD_CO][V];
#pragma unroll
    for (int co = 0; co < HEAD_CO; ++co)
#pragma unroll
      for (int k = 0; k < V; ++k) acc[co][k] = 0.f;
    for (int ci = 0; ci < Cin; ++ci) {
      float xv[V];
      Elt<T>::ldv(xp + (size_t)ci * P, xv);
#pragma unroll
      for (int co = 0; co < HEAD_CO; ++co) {
        const float wv = wl[ci * HEAD_CO + co];
#pragma unroll
        for (int k = 0; k < V; ++k) acc[co][k] = fmaf(wv, xv[k], acc[co][k]);
      }
    }
#pragma unroll
    for (int co = 0; co < HEAD_CO; ++co)
      if (co < Cout) Elt<T>::stv(y + (n * Cout + co) * P + p, acc[co]);
  }
}

// dx[n][ci][p] = sum_co w[co][ci] dy[n][co][p]
template <typename T>
__global__ __launch_bounds__(256) void k_head_bwd_data(const T* __restrict__ dy, const T* __restrict__ w,
                                                       T* __restrict__ dx, int Cin, int Cout, size_t P, size_t nvec) {
  constexpr int V = Elt<T>::V;
  extern __shared__ float wl[];
  head_load_w(w, wl, Cin, Cout);
  const size_t pv = P / V;
  for (size_t v = (size_t)blockIdx.x * 256 + threadIdx.x; v < nvec; v += (size_t)gridDim.x * 256) {
    const size_t n = v / pv, p = (v - n * pv) * V;
    float g[HEAD_CO][V];
#pragma unroll
    for (int co = 0; co < HEAD_CO; ++co) {
      if (co < Cout) {
        Elt<T>::ldv(dy + (n * Cout + co) * P + p, g[co]);
      } else {
#pragma unroll
        for (int k = 0; k < V; ++k) g[co][k] = 0.f;
      }
    }
    T* dp = dx + n * Cin * P + p;
    for (int ci = 0; ci < Cin; ++ci) {
      float o[V];
#pragma unroll
      for (int k = 0; k < V; ++k) o[k] = 0.f;
#pragma unroll
      for (int co = 0; co < HEAD_CO; ++co) {
        const float wv = wl[ci * HEAD_CO + co];
#pragma unroll
        for (int k = 0; k < V; ++k) o[k] = fmaf(wv, g[co][k], o[k]);
      }
      Elt<T>::stv(dp + (size_t)ci * P, o);
    }
  }
}

// part[blockIdx.x][co][ci] = sum over the workgroup's pixel vectors of dy[n][co][p] x[n][ci][p].  blockIdx.y picks
// a group of 64 input channels, wave j of the workgroup's four takes sixteen of them; every wave walks all of the
// workgroup's pixel vectors (64 per step), then adds its lanes' sums in a butterfly and lane 0 stores them.
template <typename T>
__global__ __launch_bounds__(256) void k_head_bwd_weight(const T* __restrict__ x, const T* __restrict__ dy,
                                                         float* __restrict__ part, int Cin, int Cout, size_t P,
                                                         size_t nvec, size_t per_block) {
  constexpr int V = Elt<T>::V;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int ci0 = blockIdx.y * 64 + wave * 16;
  const size_t pv = P / V;
  const size_t vbeg = (size_t)blockIdx.x * per_block, vend = vbeg + per_block < nvec ? vbeg + per_block : nvec;
  float acc[16][HEAD_CO];
#pragma unroll
  for (int c = 0; c < 16; ++c)
#pragma unroll
    for (int co = 0; co < HEAD_CO; ++co) acc[c][co] = 0.f;
  for (size_t v = vbeg + lane; v < vend; v += 64) {
    const size_t n = v / pv, p = (v - n * pv) * V;
    float g[HEAD_CO][V];
#pragma unroll
    for (int co = 0; co < HEAD_CO; ++co) {
      if (co < Cout) {
        Elt<T>::ldv(dy + (n * Cout + co) * P + p, g[co]);
      } else {
#pragma unroll
        for (int k = 0; k < V; ++k) g[co][k] = 0.f;
      }
    }
    const T* xp = x + n * Cin * P + p;
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      float xv[V];
      if (ci0 + c < Cin) {
        Elt<T>::ldv(xp + (size_t)(ci0 + c) * P, xv);
      } else {
#pragma unroll
        for (int k = 0; k < V; ++k) xv[k] = 0.f;
      }
#pragma unroll
      for (int co = 0; co < HEAD_CO; ++co)
#pragma unroll
        for (int k = 0; k < V; ++k) acc[c][co] = fmaf(g[co][k], xv[k], acc[c][co]);
    }
  }
  float* out = part + (size_t)blockIdx.x * Cout * Cin;
#pragma unroll
  for (int c = 0; c < 16; ++c)
#pragma unroll
    for (int co = 0; co < HEAD_CO; ++co) {
      float s = acc[c][co];
#pragma unroll
      for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m);
      if (lane == 0 && co < Cout && ci0 + c < Cin) out[(size_t)co * Cin + ci0 + c] = s;
    }
}

// The streaming head kernels apply when the vectors line up: P a multiple of the 16-byte vector, aligned tensors.
bool head_fast(int Cin, int Cout, size_t P, int bf, const void* a, const void* b) {
  return Cout <= HEAD_CO && Cin <= HEAD_CIN && P % (bf ? 8 : 4) == 0 && aligned16(a) && aligned16(b);
}
// Workgroups of the head's weight gradient: at least eight pixel vectors per lane, at most HEAD_PARTS.
int head_parts(int N, size_t P) {
  const size_t nvec = (size_t)N * P / 4;
  return (int)std::max<size_t>(1, std::min<size_t>(HEAD_PARTS, nvec / 512));
}

// Splits of the contraction for the weight gradients (K = pixels of one image): about 1024 workgroups,
// chunks of at least 64 pixels, at most 64 partial sums per image.
int pick_splitk(int tiles, int batch, int K) {
  int s = std::max(1, 1024 / std::max(1, tiles * batch));
  s = std::min(s, std::max(1, K / 64));
  return std::min(s, 64);
}

hipStream_t S(void* stream) { return static_cast<hipStream_t>(stream); }

// ---- typed bodies of the entry points (T = float, or uint16_t holding bfloat16) ----
template <typename T>
int relu_fwd_t(const T* x, T* y, size_t n, void* stream) {
  if (!x || !y) return ROTCONV_ERR_NULL;
  if (aligned16(x) && aligned16(y))
    hipLaunchKernelGGL((k_relu_fwd<T, true>), dim3(blocks_for(n / Elt<T>::V + 8)), dim3(256), 0, S(stream), x, y, n);
  else
    hipLaunchKernelGGL((k_relu_fwd<T, false>), dim3(blocks_for(n)), dim3(256), 0, S(stream), x, y, n);
  return finish();
}
template <typename T>
int relu_bwd_t(const T* y, const T* dy, T* dx, size_t n, void* stream) {
  if (!y || !dy || !dx) return ROTCONV_ERR_NULL;
  if (aligned16(y) && aligned16(dy) && aligned16(dx))
    hipLaunchKernelGGL((k_relu_bwd<T, true>), dim3(blocks_for(n / Elt<T>::V + 8)), dim3(256), 0, S(stream), y, dy, dx, n);
  else
    hipLaunchKernelGGL((k_relu_bwd<T, false>), dim3(blocks_for(n)), dim3(256), 0, S(stream), y, dy, dx, n);
  return finish();
}
template <typename T>
int maxpool2_fwd_t(const T* x, T* y, uint8_t* idx, int N, int C, int H, int W, void* stream) {
  if (!x || !y || !idx) return ROTCONV_ERR_NULL;
  if (N < 1 || C < 1 || H < 2 || W < 2 || (H & 1) || (W & 1)) return ROTCONV_ERR_SHAPE;
  const size_t planes = (size_t)N * C;
  if (W % Elt<T>::V == 0 && aligned16(x) && aligned16(y) && aligned16(idx))
    hipLaunchKernelGGL((k_maxpool2_fwd<T, true>), dim3(blocks_for(planes * H * W / (2 * Elt<T>::V))), dim3(256), 0,
                       S(stream), x, y, idx, planes, H, W);
  else
    hipLaunchKernelGGL((k_maxpool2_fwd<T, false>), dim3(blocks_for(planes * H * W / 4)), dim3(256), 0, S(stream), x, y,
                       idx, planes, H, W);
  return finish();
}
template <typename T>
int maxpool2_bwd_t(const T* dy, const uint8_t* idx, T* dx, int N, int C, int H, int W, int accumulate, void* stream) {
  if (!dy || !idx || !dx) return ROTCONV_ERR_NULL;
  if (N < 1 || C < 1 || H < 2 || W < 2 || (H & 1) || (W & 1)) return ROTCONV_ERR_SHAPE;
  const size_t planes = (size_t)N * C;
  if (W % Elt<T>::V == 0 && aligned16(dy) && aligned16(dx) && aligned16(idx))
    hipLaunchKernelGGL((k_maxpool2_bwd<T, true>), dim3(blocks_for(planes * H * W / Elt<T>::V)), dim3(256), 0, S(stream),
                       dy, idx, dx, planes, H, W, accumulate);
  else
    hipLaunchKernelGGL((k_maxpool2_bwd<T, false>), dim3(blocks_for(planes * H * W)), dim3(256), 0, S(stream), dy, idx, dx,
                       planes, H, W, accumulate);
  return finish();
}
template <typename T>
int concat2_t(const T* a, const T* b, T* out, int N, int Ca, int Cb, size_t P, void* stream) {
  if (!a || !b || !out) return ROTCONV_ERR_NULL;
  if (N < 1 || Ca < 1 || Cb < 1 || P < 1) return ROTCONV_ERR_SHAPE;
  const size_t na = (size_t)Ca * P, nb = (size_t)Cb * P;
  constexpr int V = Elt<T>::V;
  if (na % V == 0 && nb % V == 0 && aligned16(a) && aligned16(b) && aligned16(out))
    hipLaunchKernelGGL((k_concat2<T, true>), dim3(blocks_for((size_t)N * (na + nb) / V)), dim3(256), 0, S(stream), a, b,
                       out, N, na, nb);
  else
    hipLaunchKernelGGL((k_concat2<T, false>), dim3(blocks_for((size_t)N * (na + nb))), dim3(256), 0, S(stream), a, b, out,
                       N, na, nb);
  return finish();
}
template <typename T>
int split2_t(const T* dcat, T* da, T* db, int N, int Ca, int Cb, size_t P, int accumulate_a, void* stream) {
  if (!dcat || !da || !db) return ROTCONV_ERR_NULL;
  if (N < 1 || Ca < 1 || Cb < 1 || P < 1) return ROTCONV_ERR_SHAPE;
  const size_t na = (size_t)Ca * P, nb = (size_t)Cb * P;
  constexpr int V = Elt<T>::V;
  if (na % V == 0 && nb % V == 0 && aligned16(dcat) && aligned16(da) && aligned16(db))
    hipLaunchKernelGGL((k_split2<T, true>), dim3(blocks_for((size_t)N * (na + nb) / V)), dim3(256), 0, S(stream), dcat,
                       da, db, N, na, nb, accumulate_a);
  else
    hipLaunchKernelGGL((k_split2<T, false>), dim3(blocks_for((size_t)N * (na + nb))), dim3(256), 0, S(stream), dcat, da,
                       db, N, na, nb, accumulate_a);
  return finish();
}
template <typename T>
int softmax_ce_t(const T* logits, const int32_t* labels, float* loss, T* dlogits, int N, int K, size_t P, void* ws,
                 size_t ws_bytes, void* stream) {
  if (!logits || !labels || !loss || !dlogits) return ROTCONV_ERR_NULL;
  if (N < 1 || K < 1 || P < 1) return ROTCONV_ERR_SHAPE;
  if (!ws || ws_bytes < (size_t)N * P * sizeof(float)) return ROTCONV_ERR_WORKSPACE;
  const float inv = 1.0f / (float)((double)N * (double)P);
  const unsigned blocks = std::min(blocks_for((size_t)N * P), 4096u);    // one partial loss each (4 bytes of ws)
  hipLaunchKernelGGL((k_softmax_ce<T>), dim3(blocks), dim3(256), 0, S(stream), logits, labels, (float*)ws, dlogits, N,
                     K, P, inv);
  hipLaunchKernelGGL(k_mean, dim3(1), dim3(1024), 0, S(stream), (const float*)ws, loss, (size_t)blocks, inv);
  return finish();
}

// The GEMM-shaped layers.  bf = 1: x / y / dy / dx and w are bfloat16; weight gradients stay fp32.
int upconv2_fwd_g(const void* x, const void* w, void* y, int N, int Cin, int Cout, int H, int W, int bf, void* stream) {
  if (!x || !w || !y) return ROTCONV_ERR_NULL;
  if (N < 1 || Cin < 1 || Cout < 1 || H < 1 || W < 1) return ROTCONV_ERR_SHAPE;
  GemmArgs a{};
  a.M = 4 * Cout; a.N = H * W; a.K = Cin; a.lda = 4 * Cout; a.ldb = H * W; a.ldc = H * W; a.transA = 1; a.transB = 0;
  a.batch = N; a.splitk = 1; a.strideA = 0; a.strideB = (size_t)Cin * H * W; a.strideC = (size_t)Cout * 4 * H * W;
  a.shufB = 0; a.shufC = 1; a.shufH = H; a.shufW = W;
  a.bf16A = a.bf16B = a.bf16C = bf;
  launch_gemm(a, w, x, y, S(stream));
  return finish();
}
int upconv2_bwd_data_g(const void* dy, const void* w, void* dx, int N, int Cin, int Cout, int H, int W, int bf,
                       void* stream) {
  if (!dy || !w || !dx) return ROTCONV_ERR_NULL;
  if (N < 1 || Cin < 1 || Cout < 1 || H < 1 || W < 1) return ROTCONV_ERR_SHAPE;
  GemmArgs a{};
  a.M = Cin; a.N = H * W; a.K = 4 * Cout; a.lda = 4 * Cout; a.ldb = 0; a.ldc = H * W; a.transA = 0; a.transB = 0;
  a.batch = N; a.splitk = 1; a.strideA = 0; a.strideB = (size_t)Cout * 4 * H * W; a.strideC = (size_t)Cin * H * W;
  a.shufB = 1; a.shufC = 0; a.shufH = H; a.shufW = W;
  a.bf16A = a.bf16B = a.bf16C = bf;
  launch_gemm(a, w, dy, dx, S(stream));
  return finish();
}
int upconv2_bwd_weight_g(const void* x, const void* dy, float* dw, int N, int Cin, int Cout, int H, int W, void* ws,
                         size_t ws_bytes, int bf, void* stream) {
  if (!x || !dy || !dw) return ROTCONV_ERR_NULL;
  if (N < 1 || Cin < 1 || Cout < 1 || H < 1 || W < 1) return ROTCONV_ERR_SHAPE;
  if (!ws || ws_bytes < glue_upconv2_workspace_bytes(N, Cin, Cout, H, W)) return ROTCONV_ERR_WORKSPACE;
  const int tiles = ((Cin + 127) / 128) * ((4 * Cout + 127) / 128);
  GemmArgs a{};
  a.M = Cin; a.N = 4 * Cout; a.K = H * W; a.lda = H * W; a.ldb = 0; a.ldc = 4 * Cout; a.transA = 0; a.transB = 1;
  a.batch = N; a.splitk = pick_splitk(tiles, N, H * W); a.strideA = (size_t)Cin * H * W;
  a.strideB = (size_t)Cout * 4 * H * W; a.strideC = (size_t)Cin * 4 * Cout;
  a.shufB = 1; a.shufC = 0; a.shufH = H; a.shufW = W;
  a.bf16A = a.bf16B = bf;
  launch_gemm(a, x, dy, ws, S(stream));
  launch_sum_parts((const float*)ws, dw, a.strideC, N * a.splitk, a.strideC, S(stream));
  return finish();
}
int conv1x1_fwd_g(const void* x, const void* w, void* y, int N, int Cin, int Cout, size_t P, int bf, void* stream) {
  if (!x || !w || !y) return ROTCONV_ERR_NULL;
  if (N < 1 || Cin < 1 || Cout < 1 || P < 1 || P > 0x7fffffff) return ROTCONV_ERR_SHAPE;
  if (head_fast(Cin, Cout, P, bf, x, y)) {
    const size_t nvec = (size_t)N * P / (bf ? 8 : 4);
    const size_t lds = (size_t)Cin * HEAD_CO * sizeof(float);
    if (bf) hipLaunchKernelGGL(k_head_fwd<uint16_t>, dim3(blocks_for(nvec)), dim3(256), lds, S(stream), (const uint16_t*)x,
                               (const uint16_t*)w, (uint16_t*)y, Cin, Cout, P, nvec);
    else hipLaunchKernelGGL(k_head_fwd<float>, dim3(blocks_for(nvec)), dim3(256), lds, S(stream), (const float*)x,
                            (const float*)w, (float*)y, Cin, Cout, P, nvec);
    return finish();
  }
  GemmArgs a{};
  a.M = Cout; a.N = (int)P; a.K = Cin; a.lda = Cin; a.ldb = (int)P; a.ldc = (int)P; a.batch = N; a.splitk = 1;
  a.strideB = (size_t)Cin * P; a.strideC = (size_t)Cout * P;
  a.bf16A = a.bf16B = a.bf16C = bf;
  launch_gemm(a, w, x, y, S(stream));
  return finish();
}
int conv1x1_bwd_data_g(const void* dy, const void* w, void* dx, int N, int Cin, int Cout, size_t P, int bf,
                       void* stream) {
  if (!dy || !w || !dx) return ROTCONV_ERR_NULL;
  if (N < 1 || Cin < 1 || Cout < 1 || P < 1 || P > 0x7fffffff) return ROTCONV_ERR_SHAPE;
  if (head_fast(Cin, Cout, P, bf, dy, dx)) {
    const size_t nvec = (size_t)N * P / (bf ? 8 : 4);
    const size_t lds = (size_t)Cin * HEAD_CO * sizeof(float);
    if (bf) hipLaunchKernelGGL(k_head_bwd_data<uint16_t>, dim3(blocks_for(nvec)), dim3(256), lds, S(stream),
                               (const uint16_t*)dy, (const uint16_t*)w, (uint16_t*)dx, Cin, Cout, P, nvec);
    else hipLaunchKernelGGL(k_head_bwd_data<float>, dim3(blocks_for(nvec)), dim3(256), lds, S(stream), (const float*)dy,
                            (const float*)w, (float*)dx, Cin, Cout, P, nvec);
    return finish();
  }
  GemmArgs a{};
  a.M = Cin; a.N = (int)P; a.K = Cout; a.lda = Cin; a.transA = 1; a.ldb = (int)P; a.ldc = (int)P; a.batch = N;
  a.splitk = 1; a.strideB = (size_t)Cout * P; a.strideC = (size_t)Cin * P;
  a.bf16A = a.bf16B = a.bf16C = bf;
  launch_gemm(a, w, dy, dx, S(stream));
  return finish();
}
int conv1x1_bwd_weight_g(const void* x, const void* dy, float* dw, int N, int Cin, int Cout, size_t P, void* ws,
                         size_t ws_bytes, int bf, void* stream) {
  if (!x || !dy || !dw) return ROTCONV_ERR_NULL;
  if (N < 1 || Cin < 1 || Cout < 1 || P < 1 || P > 0x7fffffff) return ROTCONV_ERR_SHAPE;
  if (!ws || ws_bytes < glue_conv1x1_workspace_bytes(N, Cin, Cout, P)) return ROTCONV_ERR_WORKSPACE;
  if (head_fast(Cin, Cout, P, bf, x, dy)) {
    const size_t nvec = (size_t)N * P / (bf ? 8 : 4);
    const int parts = head_parts(N, P);
    const size_t per_block = ((nvec + parts - 1) / parts + 63) / 64 * 64;
    const dim3 grid(parts, (Cin + 63) / 64);
    if (bf) hipLaunchKernelGGL(k_head_bwd_weight<uint16_t>, grid, dim3(256), 0, S(stream), (const uint16_t*)x,
                               (const uint16_t*)dy, (float*)ws, Cin, Cout, P, nvec, per_block);
    else hipLaunchKernelGGL(k_head_bwd_weight<float>, grid, dim3(256), 0, S(stream), (const float*)x, (const float*)dy,
                            (float*)ws, Cin, Cout, P, nvec, per_block);
    launch_sum_parts((const float*)ws, dw, (size_t)Cout * Cin, parts, (size_t)Cout * Cin, S(stream));
    return finish();
  }
  const int tiles = ((Cout + 127) / 128) * ((Cin + 127) / 128);
  GemmArgs a{};
  a.M = Cout; a.N = Cin; a.K = (int)P; a.lda = (int)P; a.ldb = (int)P; a.transB = 1; a.ldc = Cin; a.batch = N;
  a.splitk = pick_splitk(tiles, N, (int)P); a.strideA = (size_t)Cout * P; a.strideB = (size_t)Cin * P;
  a.strideC = (size_t)Cout * Cin;
  a.bf16A = a.bf16B = bf;
  launch_gemm(a, dy, x, ws, S(stream));
  launch_sum_parts((const float*)ws, dw, a.strideC, N * a.splitk, a.strideC, S(stream));
  return finish();
}

}  // namespace
}  // namespace rotconv

using namespace rotconv;

extern "C" {

size_t glue_upconv2_workspace_bytes(int N, int Cin, int Cout, int H, int W) {
  const int tiles = ((Cin + 127) / 128) * ((4 * Cout + 127) / 128);
  return (size_t)N * pick_splitk(tiles, N, H * W) * Cin * 4 * Cout * sizeof(float);
}
size_t glue_conv1x1_workspace_bytes(int N, int Cin, int Cout, size_t P) {
  const int tiles = ((Cout + 127) / 128) * ((Cin + 127) / 128);
  const int parts = std::max(N * pick_splitk(tiles, N, (int)P), head_parts(N, P));   // either kernel family
  return (size_t)parts * Cout * Cin * sizeof(float);
}

// ---- fp32 ----
int glue_relu_fwd(const float* x, float* y, size_t n, void* stream) { return relu_fwd_t(x, y, n, stream); }
int glue_relu_bwd(const float* y, const float* dy, float* dx, size_t n, void* stream) {
  return relu_bwd_t(y, dy, dx, n, stream);
}
int glue_maxpool2_fwd(const float* x, float* y, uint8_t* idx, int N, int C, int H, int W, void* stream) {
  return maxpool2_fwd_t(x, y, idx, N, C, H, W, stream);
}
int glue_maxpool2_bwd(const float* dy, const uint8_t* idx, float* dx, int N, int C, int H, int W, int accumulate,
                      void* stream) {
  return maxpool2_bwd_t(dy, idx, dx, N, C, H, W, accumulate, stream);
}
int glue_upconv2_fwd(const float* x, const float* w, float* y, int N, int Cin, int Cout, int H, int W, void* stream) {
  return upconv2_fwd_g(x, w, y, N, Cin, Cout, H, W, 0, stream);
}
int glue_upconv2_bwd_data(const float* dy, const float* w, float* dx, int N, int Cin, int Cout, int H, int W,
                          void* stream) {
  return upconv2_bwd_data_g(dy, w, dx, N, Cin, Cout, H, W, 0, stream);
}
int glue_upconv2_bwd_weight(const float* x, const float* dy, float* dw, int N, int Cin, int Cout, int H, int W,
                            void* ws, size_t ws_bytes, void* stream) {
  return upconv2_bwd_weight_g(x, dy, dw, N, Cin, Cout, H, W, ws, ws_bytes, 0, stream);
}
int glue_concat2(const float* a, const float* b, float* out, int N, int Ca, int Cb, size_t P, void* stream) {
  return concat2_t(a, b, out, N, Ca, Cb, P, stream);
}
int glue_split2(const float* dcat, float* da, float* db, int N, int Ca, int Cb, size_t P, int accumulate_a,
                void* stream) {
  return split2_t(dcat, da, db, N, Ca, Cb, P, accumulate_a, stream);
}
int glue_conv1x1_fwd(const float* x, const float* w, float* y, int N, int Cin, int Cout, size_t P, void* stream) {
  return conv1x1_fwd_g(x, w, y, N, Cin, Cout, P, 0, stream);
}
int glue_conv1x1_bwd_data(const float* dy, const float* w, float* dx, int N, int Cin, int Cout, size_t P,
                          void* stream) {
  return conv1x1_bwd_data_g(dy, w, dx, N, Cin, Cout, P, 0, stream);
}
int glue_conv1x1_bwd_weight(const float* x, const float* dy, float* dw, int N, int Cin, int Cout, size_t P, void* ws,
                            size_t ws_bytes, void* stream) {
  return conv1x1_bwd_weight_g(x, dy, dw, N, Cin, Cout, P, ws, ws_bytes, 0, stream);
}
int glue_softmax_ce(const float* logits, const int32_t* labels, float* loss, float* dlogits, int N, int K, size_t P,
                    void* ws, size_t ws_bytes, void* stream) {
  return softmax_ce_t(logits, labels, loss, dlogits, N, K, P, ws, ws_bytes, stream);
}

// ---- bfloat16 tensors (uint16_t storage); weight gradients and the loss are fp32 ----
int glue_relu_fwd_bf16(const uint16_t* x, uint16_t* y, size_t n, void* stream) { return relu_fwd_t(x, y, n, stream); }
int glue_relu_bwd_bf16(const uint16_t* y, const uint16_t* dy, uint16_t* dx, size_t n, void* stream) {
  return relu_bwd_t(y, dy, dx, n, stream);
}
int glue_maxpool2_fwd_bf16(const uint16_t* x, uint16_t* y, uint8_t* idx, int N, int C, int H, int W, void* stream) {
  return maxpool2_fwd_t(x, y, idx, N, C, H, W, stream);
}
int glue_maxpool2_bwd_bf16(const uint16_t* dy, const uint8_t* idx, uint16_t* dx, int N, int C, int H, int W,
                           int accumulate, void* stream) {
  return maxpool2_bwd_t(dy, idx, dx, N, C, H, W, accumulate, stream);
}
int glue_upconv2_fwd_bf16(const uint16_t* x, const uint16_t* w, uint16_t* y, int N, int Cin, int Cout, int H, int W,
                          void* stream) {
  return upconv2_fwd_g(x, w, y, N, Cin, Cout, H, W, 1, stream);
}
int glue_upconv2_bwd_data_bf16(const uint16_t* dy, const uint16_t* w, uint16_t* dx, int N, int Cin, int Cout, int H,
                               int W, void* stream) {
  return upconv2_bwd_data_g(dy, w, dx, N, Cin, Cout, H, W, 1, stream);
}
int glue_upconv2_bwd_weight_bf16(const uint16_t* x, const uint16_t* dy, float* dw, int N, int Cin, int Cout, int H,
                                 int W, void* ws, size_t ws_bytes, void* stream) {
  return upconv2_bwd_weight_g(x, dy, dw, N, Cin, Cout, H, W, ws, ws_bytes, 1, stream);
}
int glue_concat2_bf16(const uint16_t* a, const uint16_t* b, uint16_t* out, int N, int Ca, int Cb, size_t P,
                      void* stream) {
  return concat2_t(a, b, out, N, Ca, Cb, P, stream);
}
int glue_split2_bf16(const uint16_t* dcat, uint16_t* da, uint16_t* db, int N, int Ca, int Cb, size_t P,
                     int accumulate_a, void* stream) {
  return split2_t(dcat, da, db, N, Ca, Cb, P, accumulate_a, stream);
}
int glue_conv1x1_fwd_bf16(const uint16_t* x, const uint16_t* w, uint16_t* y, int N, int Cin, int Cout, size_t P,
                          void* stream) {
  return conv1x1_fwd_g(x, w, y, N, Cin, Cout, P, 1, stream);
}
int glue_conv1x1_bwd_data_bf16(const uint16_t* dy, const uint16_t* w, uint16_t* dx, int N, int Cin, int Cout, size_t P,
                               void* stream) {
  return conv1x1_bwd_data_g(dy, w, dx, N, Cin, Cout, P, 1, stream);
}
int glue_conv1x1_bwd_weight_bf16(const uint16_t* x, const uint16_t* dy, float* dw, int N, int Cin, int Cout, size_t P,
                                 void* ws, size_t ws_bytes, void* stream) {
  return conv1x1_bwd_weight_g(x, dy, dw, N, Cin, Cout, P, ws, ws_bytes, 1, stream);
}
int glue_softmax_ce_bf16(const uint16_t* logits, const int32_t* labels, float* loss, uint16_t* dlogits, int N, int K,
                         size_t P, void* ws, size_t ws_bytes, void* stream) {
  return softmax_ce_t(logits, labels, loss, dlogits, N, K, P, ws, ws_bytes, stream);
}

}  // extern "C"
