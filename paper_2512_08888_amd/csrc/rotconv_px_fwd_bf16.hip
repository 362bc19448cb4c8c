// Pooled forward on bf16 tensors with the matrix instruction turned round: M = 16 filters, N = 16 PIXELS.
//
// v_mfma_f32_16x16x32_bf16 leaves D[m][n] in lane (m / 4, n), four consecutive m per lane.  With the filters on M and
// sixteen consecutive pixels of a row on N, a lane holds the products of FOUR filters at ONE pixel column, and the
// sixteen lanes of a DPP row are sixteen consecutive columns: the placement of Eq. 8 then needs no exchange at all,
// the products of the columns x-1 / x+1 are read by the additions themselves through a shift inside the 16-lane row
// (place_row16), as in the first-layer kernels.  On bf16 tensors the matrix pipe is 16 times faster than in fp32
// while a vector instruction costs the same, so the forward is bound by the method's R * 9 placement additions and
// the max / arg-max (Eq. 10): this layout executes them with nothing around them.  What it pays: 14 of a wave's 16
// columns are outputs (the two outer lanes of a row only supply products), on the matrix instructions too.
//
//   * a wave takes 16 consecutive slots of the padded band-row sequence (rows of W + 2 slots laid end to end, as in
//     the first-layer kernels), walks down its band of rows; the NWV waves of a workgroup take consecutive chunks and
//     share one block of 16 filters, whose Q banks are LDS-resident as ready matrix operands
//     [bank][K-step][tap][lane] x 16 bytes (lane (g, m): filter m, channels 8g .. 8g+7 of the K-step);
//   * the pixel operand of a K-step is eight bf16 values of eight consecutive channels at the lane's pixel, loaded
//     two-byte-wise (16 lanes = 32 contiguous bytes per channel), one row ahead;
//   * per bank: 9 x NKS matrix instructions into nine accumulators, then for each of the lane's four filters the
//     placement block (32 additions), the bank's maximum and its orientation, merged into the running best with the
//     smallest-index rule; fused ReLU, one two-byte value and one idx byte per lane and filter.
//
// Conditions (px_fwd_bf16_supported; taken by default only where it is the faster kernel): 3 x 3 / stride 1 / pad 1, bf16 plan, max-pool over all R = 4 Q orientations of an evenly spaced closed
// set (Q = 1, 2, 4), 8 <= Cin <= 128 with Cin % 8 == 0.
#include <algorithm>

#include "rotconv_lanepx.h"
#include "rotconv_px_fwd_bf16.h"

namespace rotconv {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));

constexpr int kOutCols = 14;     // outputs per wave and row

struct PxGeom {
  int N, Cin, H, W, Cout, TY;
  int nbr;      // bands per image
  int nfb;      // blocks of 16 filters
  int nchunk;   // 14-slot chunks of the padded band-row sequence
  int ngrp;     // groups of NWV chunks (one workgroup each, per filter block)
  long nb;      // band rows in all
};

template <int Q, int NKS, int NWV, bool RELU>
__global__ __launch_bounds__(64 * NWV, NWV == 4 ? 2 : 1) void k_px_fwd_bf16(const uint16_t* __restrict__ x, const u4* __restrict__ wt,
                                                         uint16_t* __restrict__ ypool, uint8_t* __restrict__ idx,
                                                         const PxGeom g) {
  constexpr int NOP = Q * NKS * 9;          // matrix operands of a filter block
  extern __shared__ u4 Wl[];                // [Q][NKS][9][64]
  const int tid = threadIdx.x;
  // XCD-aware order (workgroup i runs on XCD i % 8): the filter blocks of one group of pixel chunks follow one another
  // on the same XCD and share its L2 copy of the input rows
  const int nwg = g.ngrp * g.nfb, per_xcd = (nwg + 7) / 8;
  const int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (v >= nwg) return;
  const int fb = v % g.nfb, grp = v / g.nfb;
  {
    const u4* src = wt + (size_t)fb * NOP * 64;
    for (int i = tid; i < NOP * 64; i += 64 * NWV) Wl[i] = src[i];
  }
  __syncthreads();
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64;
  const int chunk = grp * NWV + wave;
  if (chunk >= g.nchunk) return;
  const int lg = lane / 16, n = lane % 16;
  const int Wp = g.W + 2;
  const long slot = (long)chunk * kOutCols + n;
  const long b = slot / Wp;
  const int xs = (int)(slot - b * Wp) - 1;        // -1 ... W
  const int nimg = (int)(b / g.nbr);
  const int y0 = (int)(b - (long)nimg * g.nbr) * g.TY;
  const bool xin = b < g.nb && xs >= 0 && xs < g.W;
  const bool outl = xin && n >= 1 && n <= kOutCols;
  const int HW = g.H * g.W;
  const unsigned xoff = xin ? (unsigned)(nimg * g.Cin * HW + xs) : 0u;
  const unsigned ooff = (unsigned)(nimg * g.Cout * HW + xs);
  // first channel of the lane's eight in every K-step (a group beyond Cin re-reads the last eight: zero weights meet them)
  unsigned coff[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) coff[ks] = (unsigned)(min(ks * 32 + lg * 8, g.Cin - 8) * HW);

  // the pixel operands of a row: [K-step] x eight bf16 (channel pairs packed low / high); outside the image: zero
  auto load_row = [&](int y, u4 (&dst)[NKS]) {
    const bool in = xin && y >= 0 && y < g.H;
    const unsigned o = in ? xoff + (unsigned)(y * g.W) : 0u;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      const uint16_t* p = x + (o + (in ? coff[ks] : 0u));
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t lo = p[(unsigned)((2 * j) * HW)], hi = p[(unsigned)((2 * j + 1) * HW)];
        dst[ks][j] = lo | (hi << 16);
      }
    }
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
      for (int j = 0; j < 4; ++j) dst[ks][j] = in ? dst[ks][j] : 0u;
  };

  float A[4][Q][4], B[4][Q][4];        // rolling placement sums: [filter of the lane][bank][quarter turn]
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int q = 0; q < Q; ++q)
#pragma unroll
      for (int s = 0; s < 4; ++s) A[k][q][s] = B[k][q][s] = 0.f;

  // with one or two banks a row is too short to cover a load from far memory: the pixel operands run two rows ahead
  constexpr bool PF2 = Q < 4;
  u4 xc[NKS], xn[NKS], xn2[NKS];
  load_row(y0 - 1, xc);
  if constexpr (PF2) load_row(y0, xn);
  const u4* wl = Wl + lane;
  const int co0 = fb * 16 + lg * 4;          // the lane's four filters
  const unsigned obase = (unsigned)(lg * 4 * HW);
  for (int t = 0; t < g.TY + 2; ++t) {
    const int h = y0 - 1 + t;                // product row
    if constexpr (PF2) load_row(h + 2, xn2);
    else load_row(h + 1, xn);
    const int yo = h - 1;                    // the output row this iteration completes
    const bool store = outl && t >= 2 && yo < g.H;
    const unsigned orow = ooff + (unsigned)(yo * g.W);
    float best[4];
    int besti[4];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
      f4 acc[9];
      u4 aw[2];
      aw[0] = wl[(q * NKS * 9) * 64];
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        const bf8 bx = __builtin_bit_cast(bf8, xc[ks]);
#pragma unroll
        for (int u = 0; u < 9; ++u) {
          const int e = ks * 9 + u;
          if (e + 1 < NKS * 9) aw[(e + 1) & 1] = wl[(q * NKS * 9 + e + 1) * 64];
          const f4 zero = f4{0.f, 0.f, 0.f, 0.f};
          acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, aw[e & 1]), bx, ks == 0 ? zero : acc[u], 0, 0, 0);
        }
      }
      // The placement block below is inline assembly: the compiler does not see that it reads matrix results, so the
      // wait between the last matrix instruction and a vector read of its result is put here by hand (this
      // instruction needs at most 11 wait states; the earlier ones are older still).
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("s_nop 15\n\ts_nop 3");
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        float P[9], o[4];
#pragma unroll
        for (int u = 0; u < 9; ++u) P[u] = acc[u][k];
        place_row16(P, A[k][q], B[k][q], o);
        // the bank's maximum and the smallest of its orientations (r = s Q + q) that attains it
        const float bv = max3(o[0], o[1], max2(o[2], o[3]));
        int bi = 3 * Q + q;
#pragma unroll
        for (int s = 2; s >= 0; --s) bi = o[s] == bv ? s * Q + q : bi;
        if (q == 0) {
          best[k] = bv;
          besti[k] = bi;
        } else {       // across banks an equal value wins only with the smaller orientation index (Eq. 10: first maximum)
          const bool take = bv > best[k] || (bv == best[k] && bi < besti[k]);
          best[k] = take ? bv : best[k];
          besti[k] = take ? bi : besti[k];
        }
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      float v = best[k];
      int bi = besti[k];
      if (RELU) {
        const bool dead = !(v > 0.f);
        v = dead ? 0.f : v;
        bi = dead ? 255 : bi;
      }
      if (store && co0 + k < g.Cout) {     // a wave-uniform plane base (the lane group's part is in obase) + the lane's offset
        const size_t cbase = (size_t)(fb * 16 + k) * HW;
        st_at(ypool + cbase, (obase + orow) * 2u, v);
        st_at(idx + cbase, obase + orow, bi);
      }
    }
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      xc[ks] = xn[ks];
      if constexpr (PF2) xn[ks] = xn2[ks];
    }
  }
}

// One thread per (filter, channel): all Q banks from the base filter(s) with fp64 coefficients, rounded to fp32 and to
// bf16 once each, written as matrix operands [filter block][bank][K-step][tap][lane (g, m)][8 channels].
template <int NS>
__global__ __launch_bounds__(256) void k_px_pack_bf16(const uint16_t* __restrict__ w, uint16_t* __restrict__ wt,
                                                      const double* __restrict__ dense, int Q, int NKS, int nfb,
                                                      int Cin, int Cout) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  const int CinPad = NKS * 32;
  if (e >= nfb * 16 * CinPad) return;
  const int ci = e % CinPad, co = e / CinPad;
  const bool in = co < Cout && ci < Cin;
  const size_t slices = (size_t)Cout * Cin;
  const uint16_t* src = w + (size_t)(in ? co * Cin + ci : 0) * 9;
  double wv[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) wv[s] = in ? (double)bf16_to_f32(src[(size_t)(s / 9) * slices * 9 + s % 9]) : 0.0;
  const int fb = co / 16, m = co % 16, ks = ci / 32, gq = (ci % 32) / 8, c8 = ci % 8;
  for (int q = 0; q < Q; ++q) {
    const double* dq = dense + (size_t)q * 9 * NS;
#pragma unroll
    for (int u = 0; u < 9; ++u) {
      double acc = 0.0;
#pragma unroll
      for (int s = 0; s < NS; ++s) acc += dq[u * NS + s] * wv[s];
      wt[(((((size_t)fb * Q + q) * NKS + ks) * 9 + u) * 64 + gq * 16 + m) * 8 + c8] = f32_to_bf16((float)acc);
    }
  }
}

int px_nks(int Cin) { return (Cin + 31) / 32; }
int px_waves(const rotconv_plan* p) {      // two workgroups per CU while their filter blocks fit LDS together
  return (size_t)p->host.Q * px_nks(p->d.Cin) * 9 * 1024 * 2 <= 150 * 1024 ? 4 : 8;
}

PxGeom px_geom(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  PxGeom g{};
  g.N = d.N; g.Cin = d.Cin; g.H = d.H; g.W = d.W; g.Cout = d.Cout;
  g.nfb = (d.Cout + 15) / 16;
  const int nwv = px_waves(p);
  const long slots_wg = 256L * (nwv == 4 ? 2 : 1);      // workgroups the chip holds at once
  // band height: the smallest (rounds of workgroups) x (TY + 2), as in the first-layer kernels
  int ty = std::min(std::max(p->opt.direct_ty, 1), d.H);
  if (p->opt.direct_ty <= 0) {
    long best = -1;
    for (int t = std::min(8, d.H); t <= std::min(64, d.H); ++t) {
      const long nb = (long)d.N * ((d.H + t - 1) / t);
      const long chunks = (nb * (d.W + 2) - 1 + kOutCols - 1) / kOutCols;
      const long wgs = ((chunks + nwv - 1) / nwv) * g.nfb;
      const long cost = ((wgs + slots_wg - 1) / slots_wg) * (t + 2);
      if (best < 0 || cost < best) { best = cost; ty = t; }
    }
  }
  g.TY = ty;
  g.nbr = (d.H + ty - 1) / ty;
  g.nb = (long)d.N * g.nbr;
  g.nchunk = (int)((g.nb * (d.W + 2) - 1 + kOutCols - 1) / kOutCols);
  g.ngrp = (g.nchunk + nwv - 1) / nwv;
  return g;
}

template <int Q, int NKS>
void launch_k(const PxGeom& g, int nwv, bool relu, const uint16_t* x, const uint16_t* wt, uint16_t* ypool, uint8_t* idx,
              hipStream_t st) {
  const size_t lds = (size_t)Q * NKS * 9 * 1024;
  const dim3 grid((unsigned)((g.ngrp * g.nfb + 7) / 8 * 8));
  auto go = [&](auto kern, int nw) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(kern, grid, dim3(64 * nw), lds, st, x, reinterpret_cast<const u4*>(wt), ypool, idx, g);
  };
  if (nwv == 4) { if (relu) go(k_px_fwd_bf16<Q, NKS, 4, true>, 4); else go(k_px_fwd_bf16<Q, NKS, 4, false>, 4); }
  else { if (relu) go(k_px_fwd_bf16<Q, NKS, 8, true>, 8); else go(k_px_fwd_bf16<Q, NKS, 8, false>, 8); }
}

template <int Q>
void launch_q(int nks, const PxGeom& g, int nwv, bool relu, const uint16_t* x, const uint16_t* wt, uint16_t* ypool,
              uint8_t* idx, hipStream_t st) {
  switch (nks) {
    case 1: launch_k<Q, 1>(g, nwv, relu, x, wt, ypool, idx, st); break;
    case 2: launch_k<Q, 2>(g, nwv, relu, x, wt, ypool, idx, st); break;
    case 3: launch_k<Q, 3>(g, nwv, relu, x, wt, ypool, idx, st); break;
    default: launch_k<Q, 4>(g, nwv, relu, x, wt, ypool, idx, st); break;
  }
}

}  // namespace

bool px_fwd_bf16_supported(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  if (p->opt.px_fwd < 0 || d.dtype != ROTCONV_BF16) return false;
  // Where it wins (measured on the stack's layers): four banks and at most 64 input channels.  Every matrix
  // instruction reads its own 1 KB weight operand from LDS (a wave has one tile of 16 pixels to use it on: the rolling
  // sums of two tiles do not fit the registers), so from 128 channels up the LDS pipe is the bound, and with one bank
  // the kernel with eight pixels per lane has less to do per output.  px_fwd = 1 takes it wherever it can run.
  if (p->opt.px_fwd == 0 && (p->host.Q != 4 || d.Cin > 64)) return false;
  if (d.k != 3 || d.stride != 1 || d.pad != 1 || d.pool_op != ROTCONV_POOL_MAX) return false;
  if (d.Cin < 8 || d.Cin > 128 || (d.Cin & 7)) return false;
  const int Q = p->host.Q;
  if (p->ng != 1 || d.R != 4 * Q || (Q != 1 && Q != 2 && Q != 4)) return false;
  for (int q = 0; q < Q; ++q)
    for (int s = 0; s < 4; ++s)
      if (p->rot_of[q * 4 + s] != s * Q + q) return false;
  const size_t lim = (size_t)1 << 31;
  if ((size_t)d.N * d.Cout * d.H * d.W * 2 >= lim || (size_t)d.N * d.Cin * d.H * d.W * 2 >= lim) return false;
  return true;
}

size_t px_fwd_bf16_pack_bytes(const rotconv_plan* p) {
  return (size_t)((p->d.Cout + 15) / 16) * p->host.Q * px_nks(p->d.Cin) * 9 * 1024;
}

void launch_px_fwd_bf16(const rotconv_plan* p, const uint16_t* x, const uint16_t* w, uint16_t* ypool, uint8_t* idx,
                        uint16_t* wt, hipStream_t st) {
  const rotconv_desc& d = p->d;
  const int Q = p->host.Q, nks = px_nks(d.Cin), nfb = (d.Cout + 15) / 16;
  const int total = nfb * 16 * nks * 32;
  if (p->B == 1)
    hipLaunchKernelGGL(k_px_pack_bf16<9>, dim3((total + 255) / 256), dim3(256), 0, st, w, wt, p->dev.fq_dense64, Q, nks,
                       nfb, d.Cin, d.Cout);
  else
    hipLaunchKernelGGL(k_px_pack_bf16<18>, dim3((total + 255) / 256), dim3(256), 0, st, w, wt, p->dev.fq_dense64, Q, nks,
                       nfb, d.Cin, d.Cout);
  const PxGeom g = px_geom(p);
  const bool relu = d.activation == ROTCONV_ACT_RELU;
  const int nwv = px_waves(p);
  switch (Q) {
    case 1: launch_q<1>(nks, g, nwv, relu, x, wt, ypool, idx, st); break;
    case 2: launch_q<2>(nks, g, nwv, relu, x, wt, ypool, idx, st); break;
    default: launch_q<4>(nks, g, nwv, relu, x, wt, ypool, idx, st); break;
  }
}

}  // namespace rotconv
