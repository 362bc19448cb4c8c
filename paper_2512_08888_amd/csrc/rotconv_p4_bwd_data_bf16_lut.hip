// Input gradient on bfloat16 tensors through the routed-gradient table (3x3 / stride 1 / pad 1, one pool group
// holding all R orientations of a filter, more banks than base banks; paper Eq. 12, 13, 15 with the expansion of
// Sec. III-D folded in).
//
// After the max-pool a (filter, pixel) of the pooled gradient carries ONE orientation r* = idx, so the gradient that
// reaches BASE tap u' of filter co at pixel p is
//     D[u'][co][p] = sum over the 3 x 3 neighbours d of G[p + d] * T[d][idx[p + d]][u']
// (T: the rotated banks' coefficients of the base taps, from the plan; row R is zero and takes every idx outside
// [0, R)), and the input gradient is ONE contraction with the base bank:
//     dX[ci][p] = sum over (co, u') of w[co][ci][u'] * D[u'][co][p].
// D is formed in fp32 on the vector ALU (table rows from LDS), rounded to bf16 once and used as the A operand of
// v_mfma_f32_16x16x32_bf16 (M = 16 pixels, N = 16 channels, K = 32 filters): one conv-equivalent of matrix work
// instead of one per quarter turn and bank.
//
// A wave owns one image row x 32 pixels x 128 input channels (two pixel tiles x eight channel blocks of
// accumulators); lane (m, kg) builds D for pixels 2 m, 2 m + 1 of the strip and filters 8 kg .. 8 kg + 7 of the
// K-step.  The base bank is re-laid so that the B operand of (K-step, tap, channel block) is one contiguous
// kilobyte, read straight from global memory (the four waves of a workgroup, four consecutive rows, read the same
// kilobytes: L1 hits); LDS holds the table only, and the main loop has no barrier.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "rotconv_bf16.h"
#include "rotconv_kernels.h"
#include "rotconv_p4.h"

namespace rotconv {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));

constexpr int NCB = 8;                 // 16-channel blocks per wave
constexpr int CIG = 16 * NCB;          // input channels per workgroup
constexpr int NWAVE = 4;               // waves (image rows) per workgroup
constexpr int NT = 64 * NWAVE;
constexpr int kLutRows = 33;           // table rows per neighbour offset in LDS: R + 1 <= 33
constexpr int KSTEP_U4 = 9 * NCB * 64; // 16-byte words of one K-step of the re-laid bank (32 filters x 9 x 128 channels)

struct RawL {            // (G, idx) of one filter on the 3 x 4 neighbourhood of the lane's two pixels, as loaded
  uint32_t gc[3];        // the two pixels (a bf16 pair)
  uint16_t gl[3], gr[3]; // left / right neighbour
  uint16_t ic[3];        // idx of the two pixels
  uint8_t il[3], ir[3];
};

__global__ __launch_bounds__(NT) void k_p4_bwd_data_bf16_lut(const uint16_t* __restrict__ gpool,
                                                             const uint8_t* __restrict__ idx,
                                                             const u4* __restrict__ wt, const float* __restrict__ lut,
                                                             uint16_t* __restrict__ dx, float* __restrict__ part,
                                                             P4BwdGeom g) {
  extern __shared__ float Tl[];        // [base bank][9][kLutRows][12]
  {
    const int R1 = g.R + 1;
    for (int i = threadIdx.x; i < g.Q * 9 * R1 * 12; i += NT) Tl[(i / (R1 * 12)) * (kLutRows * 12) + i % (R1 * 12)] = lut[i];
  }
  __syncthreads();

  const int per_xcd = (g.units + 7) / 8;
  int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (v >= g.units) return;
  // K-steps (32 filters of a base bank) [k0, k1) of this workgroup: layers with few units share the contraction out
  // over ksplit workgroups, each writing an fp32 partial dX that is added in order afterwards
  const int spb = g.CoutPad / 32;               // K-steps per base bank
  const int ksp = v % g.ksplit; v /= g.ksplit;
  const int k0 = ksp * g.kper, k1 = min(g.Q * spb, k0 + g.kper);
  const int cig = v % g.ncig; v /= g.ncig;
  const int strip = v % g.nstrip; v /= g.nstrip;
  const int rb = v % g.nrb;
  const int n = v / g.nrb;

  const int tid = threadIdx.x;
  const int wave = tid / 64, lane = tid % 64;
  const int lg = lane / 16, lc = lane % 16;
  const int h = rb * NWAVE + wave;
  const int x0 = strip * 32;
  const bool active = h < g.H;
  const int HW = g.H * g.W;

  // ---- (G, idx) neighbourhood loads: lane-only parts once; out-of-range positions read a clamped address and get
  //      the idx byte 0xff (no orientation) ----
  const int xa = x0 + 2 * lc;                  // first of the lane's two pixels (W even: in or out together)
  uint32_t offc[3], offl[3], offr[3], invc[3], inve[3];
#pragma unroll
  for (int dr = 0; dr < 3; ++dr) {
    const int row = h - 1 + dr;
    const bool rok = active && row >= 0 && row < g.H;
    const bool okc = rok && xa < g.W, okl = rok && xa >= 1 && xa - 1 < g.W, okr = rok && xa + 2 < g.W;
    const uint32_t rowoff = (uint32_t)(rok ? row : 0) * (uint32_t)g.W;
    offc[dr] = rowoff + (uint32_t)(okc ? xa : 0);
    offl[dr] = rowoff + (uint32_t)(okl ? xa - 1 : 0);
    offr[dr] = rowoff + (uint32_t)(okr ? xa + 2 : 0);
    invc[dr] = okc ? 0u : 0xffffu;
    inve[dr] = (okl ? 0u : 0xffu) | (okr ? 0u : 0xff00u);
  }
  const uint16_t* gimg = gpool + (size_t)n * g.Cout * HW;
  const uint8_t* iimg = idx + (size_t)n * g.Cout * HW;
  auto raw_load = [&](int co, RawL& r) {      // filter co of the layer (clamped by the caller)
    const uint32_t fl = (uint32_t)co * (uint32_t)HW;
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      r.gc[dr] = *reinterpret_cast<const uint32_t*>(gimg + (fl + offc[dr]));
      r.ic[dr] = *reinterpret_cast<const uint16_t*>(iimg + (fl + offc[dr]));
      r.gl[dr] = gimg[fl + offl[dr]];
      r.gr[dr] = gimg[fl + offr[dr]];
      r.il[dr] = iimg[fl + offl[dr]];
      r.ir[dr] = iimg[fl + offr[dr]];
    }
  };
  // per neighbourhood value: its gradient as fp32 (dropped for an idx outside [0, R)) and its table-row offset
  struct LutVals { float gv[3][4]; uint32_t off[3][4]; };
  auto lut_prepare = [&](const RawL& r, bool fok, int bank, LutVals& lv) {
    const uint32_t tbase = (uint32_t)bank * (9 * kLutRows * 12);
    const uint32_t finv = fok ? 0u : 0xffffffffu;
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      const uint32_t iwc = (uint32_t)r.ic[dr] | invc[dr] | finv;
      const uint32_t iwe = ((uint32_t)r.il[dr] | ((uint32_t)r.ir[dr] << 8)) | inve[dr] | finv;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t byte = c == 0 ? (iwe & 0xffu) : c == 3 ? ((iwe >> 8) & 0xffu) : ((iwc >> (8 * (c - 1))) & 0xffu);
        const uint32_t bits = c == 0 ? ((uint32_t)r.gl[dr] << 16) : c == 3 ? ((uint32_t)r.gr[dr] << 16)
                              : c == 1 ? (r.gc[dr] << 16) : (r.gc[dr] & 0xffff0000u);
        lv.gv[dr][c] = byte < (uint32_t)g.R ? __uint_as_float(bits) : 0.f;
        lv.off[dr][c] = min(byte, (uint32_t)g.R) * 12u + tbase;
      }
    }
  };
  // D of pixel b (0, 1) of one filter, nine base taps: three groups (one per neighbour row) of three table-row reads
  // and 27 multiply-adds; fences and opaque uses keep one group's reads in flight at a time (left alone the compiler
  // gathers all reads up front and every row stays live)
  auto build_pixel = [&](const LutVals& lv, int b, float (&d)[9]) {
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      f4 t0[3], t1[3];
      float t8[3];
#pragma unroll
      for (int dc = 0; dc < 3; ++dc) {
        const float* t = Tl + (dr * 3 + dc) * (kLutRows * 12) + lv.off[dr][b + dc];
        t0[dc] = *reinterpret_cast<const f4*>(t);
        t1[dc] = *reinterpret_cast<const f4*>(t + 4);
        t8[dc] = t[8];
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int dc = 0; dc < 3; ++dc) {
        const float gvc = lv.gv[dr][b + dc];
        const float tv[9] = {t0[dc][0], t0[dc][1], t0[dc][2], t0[dc][3], t1[dc][0], t1[dc][1], t1[dc][2], t1[dc][3], t8[dc]};
#pragma unroll
        for (int u = 0; u < 9; ++u) d[u] = (dr == 0 && dc == 0) ? gvc * tv[u] : d[u] + gvc * tv[u];
      }
#pragma unroll
      for (int u = 0; u < 9; ++u) asm volatile("" : "+v"(d[u]));
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  f4 acc[NCB][2];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) { acc[cb][0] = f4{0.f, 0.f, 0.f, 0.f}; acc[cb][1] = f4{0.f, 0.f, 0.f, 0.f}; }

  // this lane's 16 bytes of B operand (K-step, tap u, channel block cb): wl[(u * NCB + cb) * 64]
  const u4* wl = wt + ((size_t)cig * g.Q * spb + k0) * KSTEP_U4 + lane;

  RawL raw[2];
  auto filt = [&](int ks, int j) { return (ks % spb) * 32 + 8 * lg + j; };   // filter j of the lane in K-step ks
  raw_load(min(filt(k0, 0), g.Cout - 1), raw[0]);
  for (int ks = k0; ks < k1; ++ks) {
    const int bank = ks / spb;
    // ---- A operands of the K-step: D of the lane's eight filters, two pixels, nine taps (bf16 pairs of filters) ----
    u4 a[9][2];
#pragma unroll
    for (int jp = 0; jp < 4; ++jp) {
      float d[2][2][9];      // [filter of the pair][pixel][tap]
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int j = 2 * jp + jj;
        // the next filter's neighbourhood (of the next K-step after the last filter; the final one is loaded twice)
        const int ksn = j == 7 ? min(ks + 1, k1 - 1) : ks, jn = j == 7 ? 0 : j + 1;
        raw_load(min(filt(ksn, jn), g.Cout - 1), raw[(j + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
        LutVals lv;
        lut_prepare(raw[j & 1], filt(ks, j) < g.Cout, bank, lv);
        build_pixel(lv, 0, d[jj][0]);
        build_pixel(lv, 1, d[jj][1]);
      }
#pragma unroll
      for (int u = 0; u < 9; ++u)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          bf2 pr;
          pr[0] = (__bf16)d[0][b][u];
          pr[1] = (__bf16)d[1][b][u];
          a[u][b][jp] = __builtin_bit_cast(uint32_t, pr);
        }
    }
    // ---- the contraction of the K-step: B straight from global memory, two (tap, channel block) operands ahead ----
    const u4* wk = wl + (size_t)(ks - k0) * KSTEP_U4;
    u4 bw[3];
    bw[0] = wk[0];
    bw[1] = wk[64];
#pragma unroll
    for (int i = 0; i < 9 * NCB; ++i) {
      if (i + 2 < 9 * NCB) bw[(i + 2) % 3] = wk[(i + 2) * 64];
      __builtin_amdgcn_sched_barrier(0);
      const int u = i / NCB, cb = i % NCB;
      acc[cb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, a[u][0]), __builtin_bit_cast(bf8, bw[i % 3]), acc[cb][0], 0, 0, 0);
      acc[cb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, a[u][1]), __builtin_bit_cast(bf8, bw[i % 3]), acc[cb][1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- store: lane (lg, lc) holds channel cb*16 + lc, pixels x0 + 8 lg + 2 i + b ----
  if (!active) return;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int ci = cig * CIG + cb * 16 + lc;
    if (ci >= g.Cin) continue;
    const int px = x0 + 8 * lg;
    const size_t o = ((size_t)n * g.Cin + ci) * HW + (size_t)h * g.W + px;
    float vals[8];
#pragma unroll
    for (int jv = 0; jv < 8; ++jv) vals[jv] = acc[cb][jv % 2][jv / 2];
    if (g.ksplit > 1) {       // fp32 partial sums [ksplit][N][Cin][H][W]
      float* po = part + (size_t)ksp * g.N * g.Cin * HW + o;
#pragma unroll
      for (int jv = 0; jv < 8; ++jv)
        if (px + jv < g.W) po[jv] = vals[jv];
    } else if ((g.W & 7) == 0) {
      if (px < g.W) {
        u4 pk;
#pragma unroll
        for (int jv = 0; jv < 4; ++jv) {
          bf2 pr;
          pr[0] = (__bf16)vals[2 * jv];
          pr[1] = (__bf16)vals[2 * jv + 1];
          pk[jv] = __builtin_bit_cast(uint32_t, pr);
        }
        *reinterpret_cast<u4*>(dx + o) = pk;
      }
    } else {
#pragma unroll
      for (int jv = 0; jv < 8; ++jv)
        if (px + jv < g.W) dx[o + jv] = f32_to_bf16(vals[jv]);
    }
  }
}

// The same kernel for layers with more than 128 input channels: the D of a (filter, pixel) does not depend on the
// input channel and building it is what bounds the kernel above, so a workgroup's four waves are NCG channel groups
// of 128 x 4 / NCG rows, and the NCG waves of a row build each K-step's D together -- wave cg the filter pairs
// [cg 4/NCG, (cg+1) 4/NCG) of every lane's four -- handing it to each other through LDS in the A-operand layout
// ([tap][pixel tile][lane][filter pair]: a wave writes its words of every lane's operand, a lane reads its operand
// with one 16-byte read).  One barrier per K-step (two buffers).
template <int NCG>
__global__ __launch_bounds__(NT) void k_p4_bwd_data_bf16_lut_shared(const uint16_t* __restrict__ gpool,
                                                             const uint8_t* __restrict__ idx,
                                                             const u4* __restrict__ wt, const float* __restrict__ lut,
                                                             uint16_t* __restrict__ dx, float* __restrict__ part,
                                                             P4BwdGeom g) {
  constexpr int NR = NWAVE / NCG;      // image rows per workgroup
  constexpr int NJP = 4 / NCG;         // filter pairs of a lane's four that a wave builds
  extern __shared__ float Tl[];        // [base bank][9][kLutRows][12], then the D buffers
  typedef u4 DBuf[NR][9][2][64];       // [row][tap][pixel tile][lane]: four filter pairs
  DBuf* Dl = reinterpret_cast<DBuf*>(Tl + g.Q * 9 * kLutRows * 12);       // two buffers
  {
    const int R1 = g.R + 1;
    for (int i = threadIdx.x; i < g.Q * 9 * R1 * 12; i += NT) Tl[(i / (R1 * 12)) * (kLutRows * 12) + i % (R1 * 12)] = lut[i];
  }
  __syncthreads();

  const int per_xcd = (g.units + 7) / 8;
  int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (v >= g.units) return;
  // K-steps (32 filters of a base bank) [k0, k1) of this workgroup: layers with few units share the contraction out
  // over ksplit workgroups, each writing an fp32 partial dX that is added in order afterwards
  const int spb = g.CoutPad / 32;               // K-steps per base bank
  const int ksp = v % g.ksplit; v /= g.ksplit;
  const int k0 = ksp * g.kper, k1 = min(g.Q * spb, k0 + g.kper);
  const int cigw = v % g.ncigw; v /= g.ncigw;       // set of NCG channel groups
  const int strip = v % g.nstrip; v /= g.nstrip;
  const int rb = v % g.nrb;
  const int n = v / g.nrb;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64;
  const int lg = lane / 16, lc = lane % 16;
  const int cg = wave % NCG, rw = wave / NCG;       // the wave's channel group and row inside the workgroup
  const int cig = min(cigw * NCG + cg, g.ncig - 1); // a wave beyond the last group redoes it (and stores nothing)
  const bool cg_on = cigw * NCG + cg < g.ncig;
  const int h = rb * NR + rw;
  const int x0 = strip * 32;
  const bool active = h < g.H;
  const int HW = g.H * g.W;

  // ---- (G, idx) neighbourhood loads: lane-only parts once; out-of-range positions read a clamped address and get
  //      the idx byte 0xff (no orientation) ----
  const int xa = x0 + 2 * lc;                  // first of the lane's two pixels (W even: in or out together)
  uint32_t offc[3], offl[3], offr[3], invc[3], inve[3];
#pragma unroll
  for (int dr = 0; dr < 3; ++dr) {
    const int row = h - 1 + dr;
    const bool rok = active && row >= 0 && row < g.H;
    const bool okc = rok && xa < g.W, okl = rok && xa >= 1 && xa - 1 < g.W, okr = rok && xa + 2 < g.W;
    const uint32_t rowoff = (uint32_t)(rok ? row : 0) * (uint32_t)g.W;
    offc[dr] = rowoff + (uint32_t)(okc ? xa : 0);
    offl[dr] = rowoff + (uint32_t)(okl ? xa - 1 : 0);
    offr[dr] = rowoff + (uint32_t)(okr ? xa + 2 : 0);
    invc[dr] = okc ? 0u : 0xffffu;
    inve[dr] = (okl ? 0u : 0xffu) | (okr ? 0u : 0xff00u);
  }
  const uint16_t* gimg = gpool + (size_t)n * g.Cout * HW;
  const uint8_t* iimg = idx + (size_t)n * g.Cout * HW;
  auto raw_load = [&](int co, RawL& r) {      // filter co of the layer (clamped by the caller)
    const uint32_t fl = (uint32_t)co * (uint32_t)HW;
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      r.gc[dr] = *reinterpret_cast<const uint32_t*>(gimg + (fl + offc[dr]));
      r.ic[dr] = *reinterpret_cast<const uint16_t*>(iimg + (fl + offc[dr]));
      r.gl[dr] = gimg[fl + offl[dr]];
      r.gr[dr] = gimg[fl + offr[dr]];
      r.il[dr] = iimg[fl + offl[dr]];
      r.ir[dr] = iimg[fl + offr[dr]];
    }
  };
  // per neighbourhood value: its gradient as fp32 (dropped for an idx outside [0, R)) and its table-row offset
  struct LutVals { float gv[3][4]; uint32_t off[3][4]; };
  auto lut_prepare = [&](const RawL& r, bool fok, int bank, LutVals& lv) {
    const uint32_t tbase = (uint32_t)bank * (9 * kLutRows * 12);
    const uint32_t finv = fok ? 0u : 0xffffffffu;
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      const uint32_t iwc = (uint32_t)r.ic[dr] | invc[dr] | finv;
      const uint32_t iwe = ((uint32_t)r.il[dr] | ((uint32_t)r.ir[dr] << 8)) | inve[dr] | finv;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t byte = c == 0 ? (iwe & 0xffu) : c == 3 ? ((iwe >> 8) & 0xffu) : ((iwc >> (8 * (c - 1))) & 0xffu);
        const uint32_t bits = c == 0 ? ((uint32_t)r.gl[dr] << 16) : c == 3 ? ((uint32_t)r.gr[dr] << 16)
                              : c == 1 ? (r.gc[dr] << 16) : (r.gc[dr] & 0xffff0000u);
        lv.gv[dr][c] = byte < (uint32_t)g.R ? __uint_as_float(bits) : 0.f;
        lv.off[dr][c] = min(byte, (uint32_t)g.R) * 12u + tbase;
      }
    }
  };
  // D of pixel b (0, 1) of one filter, nine base taps: three groups (one per neighbour row) of three table-row reads
  // and 27 multiply-adds; fences and opaque uses keep one group's reads in flight at a time (left alone the compiler
  // gathers all reads up front and every row stays live)
  auto build_pixel = [&](const LutVals& lv, int b, float (&d)[9]) {
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      f4 t0[3], t1[3];
      float t8[3];
#pragma unroll
      for (int dc = 0; dc < 3; ++dc) {
        const float* t = Tl + (dr * 3 + dc) * (kLutRows * 12) + lv.off[dr][b + dc];
        t0[dc] = *reinterpret_cast<const f4*>(t);
        t1[dc] = *reinterpret_cast<const f4*>(t + 4);
        t8[dc] = t[8];
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int dc = 0; dc < 3; ++dc) {
        const float gvc = lv.gv[dr][b + dc];
        const float tv[9] = {t0[dc][0], t0[dc][1], t0[dc][2], t0[dc][3], t1[dc][0], t1[dc][1], t1[dc][2], t1[dc][3], t8[dc]};
#pragma unroll
        for (int u = 0; u < 9; ++u) d[u] = (dr == 0 && dc == 0) ? gvc * tv[u] : d[u] + gvc * tv[u];
      }
#pragma unroll
      for (int u = 0; u < 9; ++u) asm volatile("" : "+v"(d[u]));
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  f4 acc[NCB][2];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) { acc[cb][0] = f4{0.f, 0.f, 0.f, 0.f}; acc[cb][1] = f4{0.f, 0.f, 0.f, 0.f}; }

  // this lane's 16 bytes of B operand (K-step, tap u, channel block cb): wl[(u * NCB + cb) * 64]
  const u4* wl = wt + ((size_t)cig * g.Q * spb + k0) * KSTEP_U4 + lane;

  RawL raw[2];
  auto filt = [&](int ks, int j) { return (ks % spb) * 32 + 8 * lg + j; };   // filter j of the lane in K-step ks
  raw_load(min(filt(k0, 2 * cg * NJP), g.Cout - 1), raw[0]);
  for (int ks = k0; ks < k1; ++ks) {
    const int bank = ks / spb;
    // ---- the wave's share of the K-step's D: NJP filter pairs of the lane's four, two pixels, nine taps ----
    const int par = (ks - k0) & 1;
#pragma unroll
    for (int jq = 0; jq < NJP; ++jq) {
      const int jp = cg * NJP + jq;          // filter pair of the lane's eight filters
      float d[2][2][9];      // [filter of the pair][pixel][tap]
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int j = 2 * jp + jj;
        // the next filter's neighbourhood (of the next K-step after the wave's last filter; the final one is loaded twice)
        const bool lastf = jq == NJP - 1 && jj == 1;
        const int ksn = lastf ? min(ks + 1, k1 - 1) : ks;
        const int jn = lastf ? 2 * cg * NJP : j + 1;
        raw_load(min(filt(ksn, jn), g.Cout - 1), raw[(jq * 2 + jj + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
        LutVals lv;
        lut_prepare(raw[(jq * 2 + jj) & 1], filt(ks, j) < g.Cout, bank, lv);
        build_pixel(lv, 0, d[jj][0]);
        build_pixel(lv, 1, d[jj][1]);
      }
#pragma unroll
      for (int u = 0; u < 9; ++u)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          bf2 pr;
          pr[0] = (__bf16)d[0][b][u];
          pr[1] = (__bf16)d[1][b][u];
          reinterpret_cast<uint32_t*>(&Dl[par][rw][u][b][lane])[jp] = __builtin_bit_cast(uint32_t, pr);
        }
    }
    __syncthreads();
    u4 a[9][2];
#pragma unroll
    for (int u = 0; u < 9; ++u)
#pragma unroll
      for (int b = 0; b < 2; ++b) a[u][b] = Dl[par][rw][u][b][lane];
    // ---- the contraction of the K-step: B straight from global memory, two (tap, channel block) operands ahead ----
    const u4* wk = wl + (size_t)(ks - k0) * KSTEP_U4;
    u4 bw[3];
    bw[0] = wk[0];
    bw[1] = wk[64];
#pragma unroll
    for (int i = 0; i < 9 * NCB; ++i) {
      if (i + 2 < 9 * NCB) bw[(i + 2) % 3] = wk[(i + 2) * 64];
      __builtin_amdgcn_sched_barrier(0);
      const int u = i / NCB, cb = i % NCB;
      acc[cb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, a[u][0]), __builtin_bit_cast(bf8, bw[i % 3]), acc[cb][0], 0, 0, 0);
      acc[cb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, a[u][1]), __builtin_bit_cast(bf8, bw[i % 3]), acc[cb][1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- store: lane (lg, lc) holds channel cb*16 + lc, pixels x0 + 8 lg + 2 i + b ----
  if (!active || !cg_on) return;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int ci = cig * CIG + cb * 16 + lc;
    if (ci >= g.Cin) continue;
    const int px = x0 + 8 * lg;
    const size_t o = ((size_t)n * g.Cin + ci) * HW + (size_t)h * g.W + px;
    float vals[8];
#pragma unroll
    for (int jv = 0; jv < 8; ++jv) vals[jv] = acc[cb][jv % 2][jv / 2];
    if (g.ksplit > 1) {       // fp32 partial sums [ksplit][N][Cin][H][W]
      float* po = part + (size_t)ksp * g.N * g.Cin * HW + o;
#pragma unroll
      for (int jv = 0; jv < 8; ++jv)
        if (px + jv < g.W) po[jv] = vals[jv];
    } else if ((g.W & 7) == 0) {
      if (px < g.W) {
        u4 pk;
#pragma unroll
        for (int jv = 0; jv < 4; ++jv) {
          bf2 pr;
          pr[0] = (__bf16)vals[2 * jv];
          pr[1] = (__bf16)vals[2 * jv + 1];
          pk[jv] = __builtin_bit_cast(uint32_t, pr);
        }
        *reinterpret_cast<u4*>(dx + o) = pk;
      }
    } else {
#pragma unroll
      for (int jv = 0; jv < 8; ++jv)
        if (px + jv < g.W) dx[o + jv] = f32_to_bf16(vals[jv]);
    }
  }
}

// dx[e] = bf16( sum over the splits, ascending, of part[s][e] )
__global__ __launch_bounds__(256) void k_sum_dx_bf16(const float* __restrict__ part, uint16_t* __restrict__ dx, size_t n_elem,
                                                     int nparts) {
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n_elem; e += (size_t)gridDim.x * 256) {
    float v = part[e];
    for (int k = 1; k < nparts; ++k) v += part[(size_t)k * n_elem + e];
    dx[e] = f32_to_bf16(v);
  }
}

// base bank(s) (bf16, exact copies) -> [channel group][base bank][K-step of 32 filters][tap][channel block][kg][channel
// 16][8 filters]: one thread per (channel group, bank, K-step, channel block, kg, channel, filter)
__global__ __launch_bounds__(256) void k_pack_bwd_bf16_lut(const uint16_t* __restrict__ w, uint16_t* __restrict__ wt, int B,
                                                           int ncig, int spb, int Cin, int Cout) {
  const size_t total = (size_t)ncig * B * spb * NCB * 4 * 16 * 8;
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int f8 = (int)(e % 8), c16 = (int)((e / 8) % 16), kg = (int)((e / 128) % 4), cb = (int)((e / 512) % NCB);
  size_t r = e / (512 * NCB);
  const int ks = (int)(r % spb); r /= spb;
  const int b = (int)(r % B);
  const int cig = (int)(r / B);
  const int co = ks * 32 + kg * 8 + f8, ci = cig * CIG + cb * 16 + c16;
  const bool in = co < Cout && ci < Cin;
  const uint16_t* src = w + ((size_t)b * Cout * Cin + (size_t)(in ? co * Cin + ci : 0)) * 9;
  // element (tap u): 16-byte word ((cig*B + b)*spb + ks) * KSTEP_U4 + (u*NCB + cb)*64 + kg*16 + c16, halfword f8
  uint16_t* dst = wt + (((((size_t)cig * B + b) * spb + ks) * KSTEP_U4 + (size_t)cb * 64 + kg * 16 + c16) * 8 + f8);
#pragma unroll
  for (int u = 0; u < 9; ++u) dst[(size_t)u * NCB * 64 * 8] = in ? src[u] : (uint16_t)0;
}

P4BwdGeom lut_geom(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  P4BwdGeom g{};
  g.N = d.N; g.Cin = d.Cin; g.CinPad = (d.Cin + CIG - 1) / CIG * CIG; g.H = d.H; g.W = d.W; g.Cout = d.Cout;
  g.CoutPad = (d.Cout + 31) / 32 * 32; g.R = d.R; g.Q = p->B; g.ng = 1; g.lut = 1; g.px = 2;
  g.ncig = g.CinPad / CIG;
  // channel groups of a row whose waves build the D of a K-step together (the rest of the four waves: rows)
  // (two groups sharing were measured slower than two independent workgroups: 0.165 against 0.124 ms at 256 channels;
  // four groups faster: 0.162 against 0.233 ms at 1024 channels)
  g.ncg = g.ncig >= 3 ? 4 : 1;
  g.ncigw = (g.ncig + g.ncg - 1) / g.ncg;
  g.nw = NWAVE / g.ncg;                      // rows per workgroup
  g.nrb = (d.H + g.nw - 1) / g.nw;
  g.nstrip = (d.W + 31) / 32;
  g.units = d.N * g.ncigw * g.nstrip * g.nrb;
  // few units and a long contraction: share the K-steps out (at least two per workgroup; partial sums within 256 MiB)
  const int steps = g.Q * (g.CoutPad / 32);
  g.ksplit = 1;
  g.kper = steps;
  if (g.units < 512 && steps >= 4) {
    const double dx_bytes = 4.0 * d.N * d.Cin * d.H * d.W;
    const int want = std::min({steps / 2, (1024 + g.units - 1) / g.units, std::max(1, (int)(268435456.0 / dx_bytes))});
    if (want > 1) {
      g.kper = (steps + want - 1) / want;
      g.ksplit = (steps + g.kper - 1) / g.kper;
    }
  }
  g.units *= g.ksplit;
  return g;
}

}  // namespace

// 3x3 / stride 1 / pad 1, bf16 tensors, even rows, the table applies (one pool group over more banks than base banks)
bool p4_bwd_data_bf16_lut_supported(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  if (d.k != 3 || d.stride != 1 || d.pad != 1 || (d.W & 1)) return false;
  return p4_bwd_lut16_choice(p);
}

size_t p4_bwd_data_bf16_lut_pack_bytes(const rotconv_plan* p) {
  const P4BwdGeom g = lut_geom(p);
  return (size_t)g.ncig * g.Q * (g.CoutPad / 32) * KSTEP_U4 * 16;
}

size_t p4_bwd_data_bf16_lut_part_bytes(const rotconv_plan* p) {
  const P4BwdGeom g = lut_geom(p);
  return g.ksplit > 1 ? (size_t)g.ksplit * p->d.N * p->d.Cin * p->d.H * p->d.W * sizeof(float) : 0;
}

void launch_p4_pack_bwd_bf16_lut(const rotconv_plan* p, const uint16_t* w, uint16_t* wt, hipStream_t st) {
  const P4BwdGeom g = lut_geom(p);
  const int spb = g.CoutPad / 32;
  const size_t total = (size_t)g.ncig * g.Q * spb * NCB * 4 * 16 * 8;
  hipLaunchKernelGGL(k_pack_bwd_bf16_lut, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, w, wt, g.Q, g.ncig, spb,
                     g.Cin, g.Cout);
}

void launch_p4_bwd_data_bf16_lut(const rotconv_plan* p, const uint16_t* gpool, const uint8_t* idx, const uint16_t* wt,
                                 uint16_t* dx, float* part, hipStream_t st) {
  const P4BwdGeom g = lut_geom(p);
  const size_t lds_t = (size_t)g.Q * 9 * kLutRows * 12 * sizeof(float);
  const int grid = (g.units + 7) / 8 * 8;
  auto go = [&](auto kern, size_t lds) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), lds, st, gpool, idx, reinterpret_cast<const u4*>(wt), p->dev.lut_bwd, dx,
                       part, g);
  };
  const size_t lds_d = (size_t)2 * g.nw * 9 * 2 * 64 * 16;       // the shared kernels' two D buffers
  if (g.ncg == 4) go(k_p4_bwd_data_bf16_lut_shared<4>, lds_t + lds_d);
  else go(k_p4_bwd_data_bf16_lut, lds_t);
  if (g.ksplit > 1) {
    const size_t n_elem = (size_t)p->d.N * p->d.Cin * p->d.H * p->d.W;
    const unsigned blocks = (unsigned)std::max<size_t>(1, std::min<size_t>((n_elem + 255) / 256, 1u << 16));
    hipLaunchKernelGGL(k_sum_dx_bf16, dim3(blocks), dim3(256), 0, st, part, dx, n_elem, g.ksplit);
  }
}

}  // namespace rotconv
