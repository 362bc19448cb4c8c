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
// Stores at a wave-uniform base plus the lane's 32-bit byte offset (the address form that needs no per-lane 64-bit
// arithmetic; written out because the compiler folds the two into a per-lane pointer and adds per store).
__device__ __forceinline__ void st_at(float* base, unsigned byte_off, float v) {
  asm volatile("global_store_dword %0, %1, %2" ::"v"(byte_off), "v"(v), "s"(base) : "memory");
}
__device__ __forceinline__ void st_at(uint16_t* base, unsigned byte_off, float v) {
  const unsigned h = f32_to_bf16(v);
  asm volatile("global_store_short %0, %1, %2" ::"v"(byte_off), "v"(h), "s"(base) : "memory");
}
__device__ __forceinline__ void st_at(uint8_t* base, unsigned byte_off, int v) {
  asm volatile("global_store_byte %0, %1, %2" ::"v"(byte_off), "v"(v), "s"(base) : "memory");
}

// Base tap that sits at row i, column j of the 3 x 3 filter after s quarter turns (the inverse of tap_i / tap_j).
constexpr int kTapAt[4][3][3] = {{{0, 1, 2}, {3, 4, 5}, {6, 7, 8}},
                                 {{2, 5, 8}, {1, 4, 7}, {0, 3, 6}},
                                 {{8, 7, 6}, {5, 4, 3}, {2, 1, 0}},
                                 {{6, 3, 0}, {7, 4, 1}, {8, 5, 2}}};
constexpr bool tap_table_ok() {
  for (int s = 0; s < 4; ++s)
    for (int u = 0; u < 9; ++u)
      if (kTapAt[s][tap_i(s, u)][tap_j(s, u)] != u) return false;
  return true;
}
static_assert(tap_table_ok(), "kTapAt is the inverse of tap_i / tap_j");

// Placement of one product row for the four quarter turns of a bank (Eq. 8).  P[u]: the lane's nine products of row h.
// Row 2 of the turned filter completes output row h-1 (o = A + ...), row 1 continues output row h (A = B + ...), row 0
// starts output row h+1 (B = ...); column 0 takes the product of the lane to the left (wave_shr:1), column 2 the one
// to the right (wave_shl:1), read by the addition itself.  The operand numbers below are kTapAt[s][i][j] + 12.  Written
// as one block so that the order is fixed: the four orientations' chains are interleaved, and the first four
// instructions read no lane-shifted operand, so a shifted read is at least two instructions behind the write of any of
// its registers (the wait the hardware asks for between a vector write and a DPP read).
#define DPP_L "wave_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
#define DPP_R "wave_shl:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
__device__ __forceinline__ void place_row(const float (&P)[9], float (&A)[4], float (&B)[4], float (&o)[4]) {
  asm volatile(
      "v_add_f32 %0, %19, %4\n\t"
      "v_add_f32 %1, %15, %5\n\t"
      "v_add_f32 %2, %13, %6\n\t"
      "v_add_f32 %3, %17, %7\n\t"
      "v_add_f32_dpp %0, %18, %0 " DPP_L
      "v_add_f32_dpp %1, %12, %1 " DPP_L
      "v_add_f32_dpp %2, %14, %2 " DPP_L
      "v_add_f32_dpp %3, %20, %3 " DPP_L
      "v_add_f32_dpp %0, %20, %0 " DPP_R
      "v_add_f32_dpp %1, %18, %1 " DPP_R
      "v_add_f32_dpp %2, %12, %2 " DPP_R
      "v_add_f32_dpp %3, %14, %3 " DPP_R
      "v_add_f32 %4, %16, %8\n\t"
      "v_add_f32 %5, %16, %9\n\t"
      "v_add_f32 %6, %16, %10\n\t"
      "v_add_f32 %7, %16, %11\n\t"
      "v_add_f32_dpp %4, %15, %4 " DPP_L
      "v_add_f32_dpp %5, %13, %5 " DPP_L
      "v_add_f32_dpp %6, %17, %6 " DPP_L
      "v_add_f32_dpp %7, %19, %7 " DPP_L
      "v_add_f32_dpp %4, %17, %4 " DPP_R
      "v_add_f32_dpp %5, %19, %5 " DPP_R
      "v_add_f32_dpp %6, %15, %6 " DPP_R
      "v_add_f32_dpp %7, %13, %7 " DPP_R
      "v_add_f32_dpp %8, %12, %13 " DPP_L
      "v_add_f32_dpp %9, %14, %17 " DPP_L
      "v_add_f32_dpp %10, %20, %19 " DPP_L
      "v_add_f32_dpp %11, %18, %15 " DPP_L
      "v_add_f32_dpp %8, %14, %8 " DPP_R
      "v_add_f32_dpp %9, %20, %9 " DPP_R
      "v_add_f32_dpp %10, %18, %10 " DPP_R
      "v_add_f32_dpp %11, %12, %11 wave_shl:1 row_mask:0xf bank_mask:0xf bound_ctrl:1"
      : "=&v"(o[0]), "=&v"(o[1]), "=&v"(o[2]), "=&v"(o[3]), "+v"(A[0]), "+v"(A[1]), "+v"(A[2]), "+v"(A[3]), "+v"(B[0]),
        "+v"(B[1]), "+v"(B[2]), "+v"(B[3])
      : "v"(P[0]), "v"(P[1]), "v"(P[2]), "v"(P[3]), "v"(P[4]), "v"(P[5]), "v"(P[6]), "v"(P[7]), "v"(P[8]));
}
#undef DPP_L
#undef DPP_R

// maxima without the canonicalising self-maximum the compiler puts in front of fmaxf (NaN inputs are undefined here)
__device__ __forceinline__ float max2(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Packed banks: [filters padded to a multiple of FB][Q][CIN * 9 padded to a multiple of 4] floats.
template <int CIN>
constexpr int wpitch() { return (CIN * 9 + 3) / 4 * 4; }

template <typename T, int CIN, int Q, int FB, bool RELU>
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
  const unsigned ooff = (unsigned)(n * g.Cout * HW + xs);           // + co * HW + y * W
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
      if (q == Q - 1) {
        // Eq. 10: the maximum first (a tree of three-input maxima), then the smallest orientation that attains it:
        // the R - 1 equality tests do not depend on one another
        float m[R];
#pragma unroll
        for (int r = 0; r < R; ++r) m[r] = out[r];
        int n = R;
#pragma unroll
        for (; n >= 3; n -= 2) m[n - 3] = max3(m[n - 3], m[n - 2], m[n - 1]);
        float best = n == 2 ? max2(m[0], m[1]) : m[0];
        int bi = R - 1;
#pragma unroll
        for (int r = R - 2; r >= 0; --r) bi = out[r] == best ? r : bi;
        if (RELU) {     // fused ReLU: dead elements get idx 255 (no orientation)
          const bool dead = !(best > 0.f);
          best = dead ? 0.f : best;
          bi = dead ? 255 : bi;
        }
        if (store && co0 + f < g.Cout) {     // a wave-uniform channel base plus the lane's 32-bit byte offset
          const size_t cbase = (size_t)(co0 + f + zero) * HW;     // scalar arithmetic here, not 2 x FB live bases
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
void launch_q(const DirGeom& g, bool relu, const void* x, const float* wb, void* ypool, uint8_t* idx, hipStream_t st) {
  constexpr int FB = 8 / Q;
  const long waves = (long)g.nchunk * g.nfb;
  const dim3 grid((unsigned)((waves + 3) / 4));
  if (relu)
    hipLaunchKernelGGL((k_direct_fwd<T, CIN, Q, FB, true>), grid, dim3(256), 0, st, static_cast<const T*>(x), wb,
                       static_cast<T*>(ypool), idx, g);
  else
    hipLaunchKernelGGL((k_direct_fwd<T, CIN, Q, FB, false>), grid, dim3(256), 0, st, static_cast<const T*>(x), wb,
                       static_cast<T*>(ypool), idx, g);
}

template <typename T, int CIN>
void launch_c(int Q, const DirGeom& g, bool relu, const void* x, const float* wb, void* ypool, uint8_t* idx,
              hipStream_t st) {
  switch (Q) {
    case 1: launch_q<T, CIN, 1>(g, relu, x, wb, ypool, idx, st); break;
    case 2: launch_q<T, CIN, 2>(g, relu, x, wb, ypool, idx, st); break;
    default: launch_q<T, CIN, 4>(g, relu, x, wb, ypool, idx, st); break;
  }
}

template <typename T>
void launch_t(int Cin, int Q, const DirGeom& g, bool relu, const void* x, const float* wb, void* ypool, uint8_t* idx,
              hipStream_t st) {
  switch (Cin) {
    case 1: launch_c<T, 1>(Q, g, relu, x, wb, ypool, idx, st); break;
    case 2: launch_c<T, 2>(Q, g, relu, x, wb, ypool, idx, st); break;
    case 3: launch_c<T, 3>(Q, g, relu, x, wb, ypool, idx, st); break;
    default: launch_c<T, 4>(Q, g, relu, x, wb, ypool, idx, st); break;
  }
}

}  // namespace

// The kernel takes: 3 x 3, stride 1, pad 1, at most four input channels, max-pooling over ALL R orientations of a
// filter, an orientation set closed under quarter turns and numbered r = s * Q + q (evenly spaced sets) with one, two
// or four first-quadrant banks; tensors whose byte offsets fit 32 bits.  Any N, H, W, Cout, any mode.
bool direct_fwd_supported(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  if (p->opt.direct < 0) return false;
  if (d.k != 3 || d.stride != 1 || d.pad != 1 || d.Cin > 4 || d.pool_op != ROTCONV_POOL_MAX) return false;
  const int Q = p->host.Q;
  if (p->ng != 1 || d.R != 4 * Q || (Q != 1 && Q != 2 && Q != 4)) return false;
  for (int q = 0; q < Q; ++q)
    for (int s = 0; s < 4; ++s)
      if (p->rot_of[q * 4 + s] != s * Q + q) return false;
  const size_t lim = (size_t)1 << 31;
  if ((size_t)d.N * d.Cout * d.H * d.W * 4 >= lim || (size_t)d.N * d.Cin * d.H * d.W * 4 >= lim) return false;
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
  if (is16) launch_t<uint16_t>(d.Cin, Q, g, relu, x, wb, ypool, idx, st);
  else launch_t<float>(d.Cin, Q, g, relu, x, wb, ypool, idx, st);
}

}  // namespace rotconv
