// Pooled forward of layers with at most four input channels (the first layer of a network) on the vector ALU.
//
// With three input channels a per-tap channel contraction is three multiply-adds: the matrix cores have nothing to
// chew on (a 16 x 16 x 4 instruction would run a quarter empty and its result would have to travel between lanes for
// the placement), and the layer's time is the method's own R * 9 placement additions plus the stores (paper Eq. 8,
// Eq. 10; the appendix' remark that small channel x filter products are not bound by the multiplications).  This
// kernel keeps the saving of Eq. 8 - the nine per-tap products P_u = sum_ci W_q[co,ci,u] * X[ci,.] of a first-quadrant
// bank are formed once and placed for its four quarter turns - with no matrix instruction, no LDS and no barrier:
//
//   * a lane owns ONE pixel column, the 64 lanes of a wave 64 consecutive columns, and the wave walks down the rows
//     of a band.  The products of row h feed the output rows h-1, h and h+1 through two rolling partial sums per
//     orientation (registers); the products of the columns x-1 and x+1 are the neighbour lanes' registers, read by
//     the additions themselves through a whole-wave lane shift (DPP wave_shr:1 / wave_shl:1 on the source operand);
//   * so that a shift never needs a value of another wave, the rows of all bands are laid end to end as padded rows
//     of W + 2 columns (x = -1 ... W; the two outer columns are outside the image, their products are zero as the
//     convolution's padding says) and a wave takes 64 consecutive slots of that sequence, of which the inner 62 are
//     its outputs; consecutive waves overlap by two slots.  62/64 * W/(W+2) of the lanes produce an output, whatever W;
//   * the weights of the wave's FB filters are wave-uniform: scalar loads inside the row loop, one scalar operand per
//     multiply-add;
//   * max / arg-max over all R orientations of a filter in ascending orientation order (smallest index wins ties),
//     the fused ReLU, one 4-byte (2-byte for bf16 tensors) store and one idx byte per lane and filter.
//
// bf16 plans: x is widened on load, the banks were rounded to bf16 when they were packed (products of bf16 values are
// exact in fp32, the sums are fp32), the pooled value is rounded once.
#include <algorithm>

#include "rotconv_bf16.h"
#include "rotconv_direct.h"
#include "rotconv_lanepx.h"
#include "rotconv_p4_taps.h"

namespace rotconv {
namespace {

// wave-uniform reads of the packed banks go through the scalar data cache (read-only path)
typedef __attribute__((address_space(4))) const float cfloat;

constexpr int kSeg = 62;   // outputs per wave and row: 64 product columns minus the two halo lanes

struct DirGeom {
  int N, H, W, Cout, TY;
  int nbr;      // bands per image
  int nfb;      // filter blocks
  int nchunk;   // 62-slot chunks of the padded band-row sequence
  long nb;      // band rows in all: N * nbr
};

__device__ __forceinline__ float ld(const float* p) { return *p; }
__device__ __forceinline__ float ld(const uint16_t* p) { return bf16_to_f32(*p); }
// Packed banks: [filters padded to a multiple of FB][Q][CIN * 9 padded to a multiple of 4] floats.
template <int CIN>
constexpr int wpitch() { return (CIN * 9 + 3) / 4 * 4; }

// PB: every bank is pooled on its own (pool groups of the four quarter turns, Sec. V-A): Q pooled channels per filter.
template <typename T, int CIN, int Q, int FB, bool RELU, bool PB = false>
__global__ __launch_bounds__(256) void k_direct_fwd(const T* __restrict__ x, const float* __restrict__ wb,
                                                    T* __restrict__ ypool, uint8_t* __restrict__ idx, const DirGeom g) {
  constexpr int R = 4 * Q, K = FB * Q, NW = CIN * 9;
  const int lane = threadIdx.x & 63;
  const int gw = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
  const int fb = gw % g.nfb, chunk = gw / g.nfb;
  if (chunk >= g.nchunk) return;
  const int Wp = g.W + 2;
  const long slot = (long)chunk * kSeg + lane;
  const long b = slot / Wp;                       // band row
  const int xs = (int)(slot - b * Wp) - 1;        // -1 ... W
  const int n = (int)(b / g.nbr);
  const int y0 = (int)(b - (long)n * g.nbr) * g.TY;
  const bool xin = b < g.nb && xs >= 0 && xs < g.W;
  const bool outl = xin && lane >= 1 && lane <= kSeg;
  const int HW = g.H * g.W;
  const unsigned xoff = xin ? (unsigned)(n * CIN * HW + xs) : 0u;   // + ci * HW + y * W
  const unsigned ooff = (unsigned)(n * g.Cout * (PB ? Q : 1) * HW + xs);      // + pooled channel * HW + y * W
  const int co0 = fb * FB;
  cfloat* wbase = (cfloat*)wb + (size_t)co0 * Q * wpitch<CIN>();

  float A[K][4], B[K][4];
#pragma unroll
  for (int k = 0; k < K; ++k)
#pragma unroll
    for (int s = 0; s < 4; ++s) A[k][s] = B[k][s] = 0.f;

  float xv[CIN], xn[CIN];
  auto load_row = [&](int y, float (&dst)[CIN]) {   // values outside the image read element 0 and are set to 0
    const bool in = xin && y >= 0 && y < g.H;
    const unsigned o = in ? xoff + (unsigned)(y * g.W) : 0u;
#pragma unroll
    for (int ci = 0; ci < CIN; ++ci) dst[ci] = ld(x + (o + (in ? (unsigned)(ci * HW) : 0u)));
#pragma unroll
    for (int ci = 0; ci < CIN; ++ci) dst[ci] = in ? dst[ci] : 0.f;
  };
  float wc[NW], wn[NW];
  auto load_w = [&](int k, int zero, float (&dst)[NW]) {
    cfloat* wq = wbase + k * wpitch<CIN>() + zero;
#pragma unroll
    for (int i = 0; i < NW; ++i) dst[i] = wq[i];
  };
  load_row(y0 - 1, xv);
  load_w(0, 0, wc);
  for (int t = 0; t < g.TY + 2; ++t) {
    const int h = y0 - 1 + t;                     // product row
    load_row(h + 1, xn);                          // next row's values, used in the next iteration
    const int yo = h - 1;                         // the output row this iteration completes
    const bool store = outl && t >= 2 && yo < g.H;
    const unsigned orow = ooff + (unsigned)(yo * g.W);
    int zero;
    asm volatile("s_mov_b32 %0, 0" : "=s"(zero));   // an address the compiler cannot hoist: the weight loads stay here
    float out[R];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int f = k / Q, q = k % Q;
      load_w((k + 1) % K, zero, wn);              // the next (filter, bank)'s weights, one section ahead
      float P[9];
#pragma unroll
      for (int u = 0; u < 9; ++u) {
        float p = wc[u] * xv[0];
#pragma unroll
        for (int ci = 1; ci < CIN; ++ci) p = fmaf(wc[ci * 9 + u], xv[ci], p);
        P[u] = p;
      }
      float o[4];
      place_row(P, A[k], B[k], o);
#pragma unroll
      for (int s = 0; s < 4; ++s) out[s * Q + q] = o[s];
      if (PB || q == Q - 1) {
        // Eq. 10: the maximum first (a tree of three-input maxima), then the smallest orientation that attains it:
        // the equality tests do not depend on one another.  PB: the group is this bank's four quarter turns.
        constexpr int NC = PB ? 4 : R;             // candidates; candidate j is orientation (PB ? j * Q + q : j)
        float m[NC], cand[NC];
#pragma unroll
        for (int j = 0; j < NC; ++j) m[j] = cand[j] = PB ? o[j] : out[j];
        int n = NC;
#pragma unroll
        for (; n >= 3; n -= 2) m[n - 3] = max3(m[n - 3], m[n - 2], m[n - 1]);
        float best = n == 2 ? max2(m[0], m[1]) : m[0];
        int bi = PB ? (NC - 1) * Q + q : NC - 1;
#pragma unroll
        for (int j = NC - 2; j >= 0; --j) bi = cand[j] == best ? (PB ? j * Q + q : j) : bi;
        if (RELU) {     // fused ReLU: dead elements get idx 255 (no orientation)
          const bool dead = !(best > 0.f);
          best = dead ? 0.f : best;
          bi = dead ? 255 : bi;
        }
        if (store && co0 + f < g.Cout) {     // a wave-uniform channel base plus the lane's 32-bit byte offset
          const size_t cbase = (size_t)((co0 + f + zero) * (PB ? Q : 1) + (PB ? q : 0)) * HW;     // scalar arithmetic, in the loop
          st_at(ypool + cbase, orow * (unsigned)sizeof(T), best);
          st_at(idx + cbase, orow, bi);
        }
      }
#pragma unroll
      for (int i = 0; i < NW; ++i) {
        asm volatile("" ::"s"(wn[i]));            // the loads issued at the head of this section land inside it
        wc[i] = wn[i];
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int ci = 0; ci < CIN; ++ci) xv[ci] = xn[ci];
  }
}

// One thread per (filter, bank, channel): its nine taps of the first-quadrant bank from the base bank(s) (Eq. 5,
// Eq. 17 / the plan's expansion table).  bf16 plans: the combination in fp64, rounded to fp32 and to bf16 once each,
// as every kernel of a bf16 plan forms its banks.
__global__ __launch_bounds__(256) void k_direct_pack(const void* __restrict__ w, float* __restrict__ wb,
                                                     const int32_t* __restrict__ fq_src,
                                                     const float* __restrict__ fq_coef,
                                                     const double* __restrict__ fq_coef64, int Q, int Cin, int Cout,
                                                     int CoutPad, int pitch, int is16) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  const int npc = Cin + 1;                        // threads per (filter, bank): the last one clears the row's pad
  if (e >= CoutPad * Q * npc) return;
  const int ci = e % npc, q = (e / npc) % Q, co = e / (npc * Q);
  float* dst = wb + (size_t)(co * Q + q) * pitch;
  if (ci >= Cin) {
    for (int i = Cin * 9; i < pitch; ++i) dst[i] = 0.f;
    return;
  }
  const bool in = co < Cout;
  const int slices = Cout * Cin;
  const size_t base = (size_t)(in ? co * Cin + ci : 0) * 9;
  for (int u = 0; u < 9; ++u) {
    float acc = 0.f;
    double a64 = 0.0;
    for (int z = 0; z < kMaxNnz; ++z) {
      const int s = fq_src[(q * 9 + u) * kMaxNnz + z];
      if (!in || s < 0) continue;
      const size_t o = base + (size_t)(s / 9) * slices * 9 + s % 9;
      if (is16) a64 += fq_coef64[(q * 9 + u) * kMaxNnz + z] * (double)bf16_to_f32(static_cast<const uint16_t*>(w)[o]);
      else acc += fq_coef[(q * 9 + u) * kMaxNnz + z] * static_cast<const float*>(w)[o];
    }
    dst[ci * 9 + u] = is16 ? bf16_to_f32(f32_to_bf16((float)a64)) : acc;
  }
}

// ---- weight gradient of such layers with a single bank (R = 4 exact quarter turns) -------------------------------
// dF[co,ci,u] = sum_pixels D_u[co,p] * X[ci,p],  D_u[co,p] = sum_s Delta_s[co, p - off_s(u)],  Delta_s = G * 1[idx == s]
// (Eq. 12, 14, and Eq. 16's inverse rotation moved in front of the contraction: the routed gradients of the four
// quarter turns are summed at the rotated tap positions first).  Same decomposition as the forward: a lane owns one
// pixel column of the padded band-row sequence and walks down a band; a (G, idx) row is routed once into four values
// that stay in registers while the row serves as h-1, h and h+1 (the row loop is unrolled three deep, the roles rotate
// by renaming); the column neighbours are the adjacent lanes' registers, read by the additions through a wave shift.
// 27 accumulators per filter and lane, added across the wave's lanes at the end of the band in a fixed order, one
// partial sum per wave; k_direct_dw_finish adds the partial sums in ascending order and applies the transposed
// first-quadrant table.  No atomics: bitwise reproducible.
constexpr int kDwFB = 2;       // filters per wave

struct DirWGeom {
  int N, H, W, Cout, CoutPad, TY, nbr, nfb, nchunk;
  long nb;
};

// the value the lane to the left (x - 1) / to the right (x + 1) holds; the wave's first / last lane gets 0.  Each use
// below is the only use of its shifted value, so the compiler folds the shift into the addition.
__device__ __forceinline__ float from_left(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x138, 0xf, 0xf, true));
}
__device__ __forceinline__ float from_right(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x130, 0xf, 0xf, true));
}

template <int CTRL, int ROWMASK>
__device__ __forceinline__ float add_dpp(float acc, float v) {
  return acc + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROWMASK, 0xf, true));
}
// sum over the 64 lanes, in lanes 48..63 (fixed order)
__device__ __forceinline__ float wave_sum(float v) {
  v = add_dpp<0xb1, 0xf>(v, v);      // quad_perm [1,0,3,2]
  v = add_dpp<0x4e, 0xf>(v, v);      // quad_perm [2,3,0,1]
  v = add_dpp<0x141, 0xf>(v, v);     // row_half_mirror
  v = add_dpp<0x140, 0xf>(v, v);     // row_mirror: every lane holds its row's sum
  v = add_dpp<0x142, 0xa>(v, v);     // row_bcast:15 into rows 1 and 3
  v = add_dpp<0x143, 0xc>(v, v);     // row_bcast:31 into rows 2 and 3
  return v;
}

template <typename T, int CIN>
__global__ __launch_bounds__(256) void k_direct_bwd_weight(const T* __restrict__ x, const T* __restrict__ gpool,
                                                           const uint8_t* __restrict__ idx, float* __restrict__ part,
                                                           const DirWGeom g) {
  constexpr int FB = kDwFB, NA = CIN * 9;
  const int lane = threadIdx.x & 63;
  const int gw = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
  const int fb = gw % g.nfb, chunk = gw / g.nfb;
  if (chunk >= g.nchunk) return;
  const int Wp = g.W + 2;
  const long slot = (long)chunk * kSeg + lane;
  const long b = slot / Wp;
  const int xs = (int)(slot - b * Wp) - 1;
  const int n = (int)(b / g.nbr);
  const int y0 = (int)(b - (long)n * g.nbr) * g.TY;
  const bool xin = b < g.nb && xs >= 0 && xs < g.W;
  const bool own = xin && lane >= 1 && lane <= kSeg;      // the lanes whose D is complete: only they accumulate
  const int HW = g.H * g.W;
  const int co0 = fb * FB;
  const unsigned xoff = xin ? (unsigned)(n * CIN * HW + xs) : 0u;
  unsigned goff[FB];
#pragma unroll
  for (int f = 0; f < FB; ++f) goff[f] = xin ? (unsigned)((n * g.Cout + min(co0 + f, g.Cout - 1)) * HW + xs) : 0u;

  float acc[FB][NA];
#pragma unroll
  for (int f = 0; f < FB; ++f)
#pragma unroll
    for (int i = 0; i < NA; ++i) acc[f][i] = 0.f;

  struct Routed { float m[FB][4]; };
  // (G, idx) of row y, routed: m[f][s] = G where idx == s, else 0 (rows outside the image, columns outside it and
  // filters beyond Cout give zeros)
  auto load_route = [&](int y, Routed& r) {
    const bool in = xin && y >= 0 && y < g.H;
    float gv[FB];
    int iv[FB];
#pragma unroll
    for (int f = 0; f < FB; ++f) {
      const unsigned o = in ? goff[f] + (unsigned)(y * g.W) : 0u;
      gv[f] = ld(gpool + o);
      iv[f] = idx[o];
    }
#pragma unroll
    for (int f = 0; f < FB; ++f) {
      const bool ok = in && co0 + f < g.Cout;
#pragma unroll
      for (int s = 0; s < 4; ++s) r.m[f][s] = (ok && iv[f] == s) ? gv[f] : 0.f;
    }
  };
  auto load_x = [&](int y, float (&dst)[CIN]) {
    const bool in = own && y >= 0 && y < g.H;
    const unsigned o = in ? xoff + (unsigned)(y * g.W) : 0u;
#pragma unroll
    for (int ci = 0; ci < CIN; ++ci) dst[ci] = ld(x + (o + (in ? (unsigned)(ci * HW) : 0u)));
#pragma unroll
    for (int ci = 0; ci < CIN; ++ci) dst[ci] = in ? dst[ci] : 0.f;
  };
  // D of row h from the routed rows h-1 (up), h (mid), h+1 (dn), times X of row h
  auto accumulate = [&](const Routed& up, const Routed& mid, const Routed& dn, const float (&xv)[CIN]) {
#pragma unroll
    for (int f = 0; f < FB; ++f) {
#pragma unroll
      for (int u = 0; u < 9; ++u) {
        float d = 0.f;
        bool first = true;
        // plain terms first, so that a lane-shifted term always meets a plain register in its addition
#pragma unroll
        for (int pass = 0; pass < 2; ++pass)
#pragma unroll
          for (int s = 0; s < 4; ++s) {
            const int i = tap_i(s, u), j = tap_j(s, u);
            if ((j == 1) != (pass == 0)) continue;
            const float mv = i == 0 ? dn.m[f][s] : i == 1 ? mid.m[f][s] : up.m[f][s];     // row h - (i - 1)
            const float t = j == 0 ? from_right(mv) : j == 2 ? from_left(mv) : mv;        // column x - (j - 1)
            d = first ? t : d + t;
            first = false;
          }
#pragma unroll
        for (int ci = 0; ci < CIN; ++ci) acc[f][ci * 9 + u] = fmaf(d, xv[ci], acc[f][ci * 9 + u]);
      }
    }
  };

  Routed ra, rb, rc;
  float xa[CIN], xb[CIN], xc[CIN];
  // rows y0-1 and y0 are routed before the loop; iteration t brings row y0 + t + 1 and finishes D row y0 + t
  load_route(y0 - 1, ra);
  load_route(y0, rb);
  load_x(y0, xa);
  const int rows = min(g.TY, g.H - y0);
  for (int t = 0; t < rows; t += 3) {
    load_route(y0 + t + 1, rc);
    load_x(y0 + t + 1, xb);
    accumulate(ra, rb, rc, xa);
    if (t + 1 < rows) {
      load_route(y0 + t + 2, ra);
      load_x(y0 + t + 2, xc);
      accumulate(rb, rc, ra, xb);
    }
    if (t + 2 < rows) {
      load_route(y0 + t + 3, rb);
      load_x(y0 + t + 3, xa);
      accumulate(rc, ra, rb, xc);
    }
  }
  float* dst = part + ((size_t)chunk * g.CoutPad + co0) * NA;
#pragma unroll
  for (int f = 0; f < FB; ++f)
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      const float sum = wave_sum(acc[f][i]);
      if (lane == 63) dst[f * NA + i] = sum;
    }
}

// dw[b][co][ci][ub] = sum_z coef_z * (sum over the waves' partial sums, ascending, of dF[co][ci][t_z]): the partial
// sums of eight interleaved groups are added by eight threads and combined in a fixed tree, then the transposed
// first-quadrant table (Eq. 16 / the adjoint of Eq. 17) is applied.  One workgroup per (filter, channel).
__global__ __launch_bounds__(256) void k_direct_dw_finish(const float* __restrict__ part, float* __restrict__ dw,
                                                          const int32_t* __restrict__ fqt_ptr,
                                                          const int32_t* __restrict__ fqt_col,
                                                          const float* __restrict__ fqt_coef, int B, int Cout, int Cin,
                                                          int CoutPad, int nchunk) {
  __shared__ float red[16][9];
  __shared__ float tot[9];
  const int co = blockIdx.x / Cin, ci = blockIdx.x % Cin;
  const int t = threadIdx.x % 16, grp = threadIdx.x / 16;      // 16 groups x (9 taps used of 16)
  const int NA = Cin * 9;
  if (t < 9) {
    float s = 0.f;
    for (int c = grp; c < nchunk; c += 16) s += part[((size_t)c * CoutPad + co) * NA + ci * 9 + t];
    red[grp][t] = s;
  }
  __syncthreads();
  if (threadIdx.x < 9) {
    const int u = threadIdx.x;
    float a[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) a[i] = red[i][u];
#pragma unroll
    for (int n = 8; n >= 1; n /= 2)
#pragma unroll
      for (int i = 0; i < n; ++i) a[i] = a[i] + a[i + n];
    tot[u] = a[0];
  }
  __syncthreads();
  if (threadIdx.x < B * 9) {
    const int b = threadIdx.x / 9, ub = threadIdx.x % 9;
    float v = 0.f;
    for (int z = fqt_ptr[b * 9 + ub]; z < fqt_ptr[b * 9 + ub + 1]; ++z) v += fqt_coef[z] * tot[fqt_col[z]];     // col = tap (one bank)
    dw[((size_t)(b * Cout + co) * Cin + ci) * 9 + ub] = v;
  }
}

DirWGeom direct_wgeom(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  DirWGeom g{};
  g.N = d.N; g.H = d.H; g.W = d.W; g.Cout = d.Cout;
  g.nfb = (d.Cout + kDwFB - 1) / kDwFB;
  g.CoutPad = g.nfb * kDwFB;
  // band height: as for the forward (measured: 32 rows on 512 x 512 x 64 filters, where this picks 32)
  int ty = std::min(std::max(p->opt.direct_ty, 1), d.H);
  if (p->opt.direct_ty <= 0) {
    long best = -1;
    for (int t = std::min(8, d.H); t <= std::min(128, d.H); ++t) {
      const long nb = (long)d.N * ((d.H + t - 1) / t);
      const long waves = ((nb * (d.W + 2) - 1 + kSeg - 1) / kSeg) * g.nfb;
      const long cost = ((waves + 1023) / 1024) * (t + 2);
      if (best < 0 || cost < best) { best = cost; ty = t; }
    }
  }
  g.TY = ty;
  g.nbr = (d.H + ty - 1) / ty;
  g.nb = (long)d.N * g.nbr;
  g.nchunk = (int)((g.nb * (d.W + 2) - 1 + kSeg - 1) / kSeg);
  return g;
}

template <typename T>
void launch_w(int Cin, const DirWGeom& g, const void* x, const void* gpool, const uint8_t* idx, float* part,
              hipStream_t st) {
  const dim3 grid((unsigned)(((long)g.nchunk * g.nfb + 3) / 4));
  const T* xp = static_cast<const T*>(x);
  const T* gp = static_cast<const T*>(gpool);
  switch (Cin) {
    case 1: hipLaunchKernelGGL((k_direct_bwd_weight<T, 1>), grid, dim3(256), 0, st, xp, gp, idx, part, g); break;
    case 2: hipLaunchKernelGGL((k_direct_bwd_weight<T, 2>), grid, dim3(256), 0, st, xp, gp, idx, part, g); break;
    case 3: hipLaunchKernelGGL((k_direct_bwd_weight<T, 3>), grid, dim3(256), 0, st, xp, gp, idx, part, g); break;
    default: hipLaunchKernelGGL((k_direct_bwd_weight<T, 4>), grid, dim3(256), 0, st, xp, gp, idx, part, g); break;
  }
}

int direct_fb(int Q) { return 8 / Q; }            // filters per wave: eight (filter, bank) pairs

int direct_pitch(int Cin) { return (Cin * 9 + 3) / 4 * 4; }

DirGeom direct_geom(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  DirGeom g{};
  g.N = d.N; g.H = d.H; g.W = d.W; g.Cout = d.Cout;
  g.nfb = (d.Cout + direct_fb(p->host.Q) - 1) / direct_fb(p->host.Q);
  // Rows per band: a band of TY rows forms TY + 2 rows of products, so long bands waste the least; but the chip's
  // 1024 SIMDs hold all waves of these launches at once, and the launch ends when the SIMD with the most waves does:
  // the band height with the smallest (waves per SIMD, rounded up) x (TY + 2).
  int ty = std::min(std::max(p->opt.direct_ty, 1), d.H);
  if (p->opt.direct_ty <= 0) {
    long best = -1;
    for (int t = std::min(8, d.H); t <= std::min(64, d.H); ++t) {
      const long nb = (long)d.N * ((d.H + t - 1) / t);
      const long waves = ((nb * (d.W + 2) - 1 + kSeg - 1) / kSeg) * g.nfb;
      const long cost = ((waves + 1023) / 1024) * (t + 2);
      if (best < 0 || cost < best) { best = cost; ty = t; }
    }
  }
  g.TY = ty;
  g.nbr = (d.H + ty - 1) / ty;
  g.nb = (long)d.N * g.nbr;
  g.nchunk = (int)((g.nb * (d.W + 2) - 1 + kSeg - 1) / kSeg);
  return g;
}

template <typename T, int CIN, int Q>
void launch_q(const DirGeom& g, bool relu, bool pb, const void* x, const float* wb, void* ypool, uint8_t* idx,
              hipStream_t st) {
  constexpr int FB = 8 / Q;
  const long waves = (long)g.nchunk * g.nfb;
  const dim3 grid((unsigned)((waves + 3) / 4));
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, grid, dim3(256), 0, st, static_cast<const T*>(x), wb, static_cast<T*>(ypool), idx, g);
  };
  if (Q > 1 && pb) { if (relu) go(k_direct_fwd<T, CIN, Q, FB, true, (Q > 1)>); else go(k_direct_fwd<T, CIN, Q, FB, false, (Q > 1)>); }
  else { if (relu) go(k_direct_fwd<T, CIN, Q, FB, true, false>); else go(k_direct_fwd<T, CIN, Q, FB, false, false>); }
}

template <typename T, int CIN>
void launch_c(int Q, const DirGeom& g, bool relu, bool pb, const void* x, const float* wb, void* ypool, uint8_t* idx,
              hipStream_t st) {
  switch (Q) {
    case 1: launch_q<T, CIN, 1>(g, relu, pb, x, wb, ypool, idx, st); break;
    case 2: launch_q<T, CIN, 2>(g, relu, pb, x, wb, ypool, idx, st); break;
    default: launch_q<T, CIN, 4>(g, relu, pb, x, wb, ypool, idx, st); break;
  }
}

template <typename T>
void launch_t(int Cin, int Q, const DirGeom& g, bool relu, bool pb, const void* x, const float* wb, void* ypool,
              uint8_t* idx, hipStream_t st) {
  switch (Cin) {
    case 1: launch_c<T, 1>(Q, g, relu, pb, x, wb, ypool, idx, st); break;
    case 2: launch_c<T, 2>(Q, g, relu, pb, x, wb, ypool, idx, st); break;
    case 3: launch_c<T, 3>(Q, g, relu, pb, x, wb, ypool, idx, st); break;
    default: launch_c<T, 4>(Q, g, relu, pb, x, wb, ypool, idx, st); break;
  }
}

}  // namespace

// The kernel takes: 3 x 3, stride 1, pad 1, at most four input channels, max-pooling over ALL R orientations of a
// filter or over the four quarter turns of each bank (pool groups of four), an orientation set closed under quarter
// turns and numbered r = s * Q + q (evenly spaced sets) with one, two or four first-quadrant banks; tensors whose byte
// offsets fit 32 bits.  Any N, H, W, Cout, any mode.
bool direct_fwd_supported(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  if (p->opt.direct < 0) return false;
  if (d.k != 3 || d.stride != 1 || d.pad != 1 || d.Cin > 4 || d.pool_op != ROTCONV_POOL_MAX) return false;
  const int Q = p->host.Q;
  if ((p->ng != 1 && p->ng != Q) || d.R != 4 * Q || (Q != 1 && Q != 2 && Q != 4)) return false;
  for (int q = 0; q < Q; ++q)
    for (int s = 0; s < 4; ++s)
      if (p->rot_of[q * 4 + s] != s * Q + q) return false;
  const size_t lim = (size_t)1 << 31;
  if ((size_t)d.N * d.Cout * p->ng * d.H * d.W * 4 >= lim || (size_t)d.N * d.Cin * d.H * d.W * 4 >= lim) return false;
  return true;
}

size_t direct_fwd_pack_floats(const rotconv_plan* p) {
  const int fb = direct_fb(p->host.Q);
  const int CoutPad = (p->d.Cout + fb - 1) / fb * fb;
  return (size_t)CoutPad * p->host.Q * direct_pitch(p->d.Cin);
}

void launch_direct_fwd(const rotconv_plan* p, const void* x, const void* w, void* ypool, uint8_t* idx, float* wb,
                       hipStream_t st) {
  const rotconv_desc& d = p->d;
  const int Q = p->host.Q, fb = direct_fb(Q), pitch = direct_pitch(d.Cin);
  const int CoutPad = (d.Cout + fb - 1) / fb * fb;
  const bool is16 = d.dtype == ROTCONV_BF16;
  const int total = CoutPad * Q * (d.Cin + 1);
  hipLaunchKernelGGL(k_direct_pack, dim3((total + 255) / 256), dim3(256), 0, st, w, wb, p->dev.fq_src, p->dev.fq_coef,
                     p->dev.fq_coef64, Q, d.Cin, d.Cout, CoutPad, pitch, is16 ? 1 : 0);
  const DirGeom g = direct_geom(p);
  const bool relu = d.activation == ROTCONV_ACT_RELU;
  const bool pb = p->ng > 1;       // pool groups of four quarter turns: every bank pooled on its own
  if (is16) launch_t<uint16_t>(d.Cin, Q, g, relu, pb, x, wb, ypool, idx, st);
  else launch_t<float>(d.Cin, Q, g, relu, pb, x, wb, ypool, idx, st);
}

}  // namespace rotconv

namespace rotconv {

// The weight gradient on the vector ALU: the forward's conditions with a single first-quadrant bank (R = 4), fp32
// plans.  With several banks the table kernels on the matrix cores execute fewer instructions, and on bf16 tensors
// the bf16 matrix-core kernel is the faster one (measured on 4 x 3 x 512 x 512 -> 64: 0.139 against 0.173 ms).
bool direct_bwd_weight_supported(const rotconv_plan* p) {
  return direct_fwd_supported(p) && p->host.Q == 1 && p->d.dtype == ROTCONV_F32;
}

size_t direct_bwd_weight_ws_floats(const rotconv_plan* p) {
  const DirWGeom g = direct_wgeom(p);
  return (size_t)g.nchunk * g.CoutPad * p->d.Cin * 9;
}

void launch_direct_bwd_weight(const rotconv_plan* p, const void* x, const void* gpool, const uint8_t* idx, float* part,
                              float* dw, hipStream_t st) {
  const rotconv_desc& d = p->d;
  const DirWGeom g = direct_wgeom(p);
  if (d.dtype == ROTCONV_BF16) launch_w<uint16_t>(d.Cin, g, x, gpool, idx, part, st);
  else launch_w<float>(d.Cin, g, x, gpool, idx, part, st);
  hipLaunchKernelGGL(k_direct_dw_finish, dim3(d.Cout * d.Cin), dim3(256), 0, st, part, dw, p->dev.fqt_ptr,
                     p->dev.fqt_col, p->dev.fqt_coef, p->B, d.Cout, d.Cin, g.CoutPad, g.nchunk);
}

}  // namespace rotconv
