// Fast input-gradient kernel for 3x3, stride 1, pad 1 (fp32), fused with the
// orientation max-pool backward (paper Eq. 12, 13, 15 in shared-product form).
//
//   dX[ci,h,x] = sum_q sum_u sum_co F_q[co,ci,u] * D^q_u[co,h,x]
//   D^q_u[co,h,x] = sum_s Delta_(q,s)[co, h+1-i_s(u), x+1-j_s(u)],   (i_s,j_s) = R_s(u)
//   Delta_r = G * 1[idx == r]
//
// i.e. the routed gradients of the four quarter turns of a bank are first summed
// at the rotated tap positions (pure selects and adds on the VALU, done on the fly
// in the MFMA A-operand layout, never stored), then ONE contraction over
// (filter, tap) runs on the fp32 matrix cores: the multiplications are shared by
// the four rotations exactly as in the forward pass.
//
// A wave owns one image row x 16 PX pixels x 64 input channels (PX = 2 or 4 pixels
// per lane, four 16x16 accumulator tiles per 16-pixel block).  Per K-step of 4
// filters a lane reads the 3 x (PX + 2) pixel neighbourhood of (G, idx) of its
// filter straight from global memory (L1/L2 resident: the waves of a
// workgroup take consecutive rows), builds its 9 PX A values and feeds
// 36 PX MFMAs.  The weights stream through LDS in chunks of 16 filters,
// double-buffered, a quarter chunk per pipeline stage, one barrier per chunk.
// A workgroup is NW waves = NW consecutive rows.  The per-bank variant runs four-wave workgroups, two per CU:
// the waves of one workgroup meet at the chunk barrier in step (the two waves of a SIMD would otherwise reach it
// one after the other, each running alone for a while), the other workgroup's waves fill the gap.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>

#include "rotconv_bf16.h"
#include "rotconv_kernels.h"
#include "rotconv_p4.h"

namespace rotconv {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int NCB = 4;                 // 16-channel blocks per wave
constexpr int CIG = 16 * NCB;          // input channels per workgroup
constexpr int WROW = 9 * CIG + 16;     // LDS floats per filter row (padded)
constexpr int WROW_TIGHT = 9 * CIG + 4; // the same for the four-wave table variant (two workgroups must fit 160 KB)
constexpr int CHUNK = 16;              // filters per LDS chunk
constexpr int kLutRows = 33;           // table rows per neighbour offset in LDS: R + 1 <= 33
constexpr int kLutRowsTight = 17;      // the four-wave table variant: R <= 16

__device__ __host__ constexpr int tap_i(int s, int u) {
  return s == 0 ? u / 3 : s == 1 ? 2 - u % 3 : s == 2 ? 2 - u / 3 : u % 3;
}
__device__ __host__ constexpr int tap_j(int s, int u) {
  return s == 0 ? u % 3 : s == 1 ? u / 3 : s == 2 ? 2 - u % 3 : 2 - u / 3;
}

template <int PX>
struct Raw {           // (G, idx) of one filter on a 3 x (PX + 2) pixel neighbourhood, as loaded
  float gc[3][PX];     // the lane's PX pixels
  float ge[3];         // first lane of a 16-lane row: the pixel left of its pixels; last lane: the pixel right of them
  uint32_t ic[3], ie[3];   // idx of the same positions (ic: PX bytes)
  uint32_t finv;       // all ones if the lane's filter of this K-step is beyond Cout
};

// Left / right neighbour values of a lane's pixels: the adjacent lane of the 16-lane row holds them (its last / first
// pixel); only the row's first and last lane take the value they loaded themselves (a shift inside the row leaves the
// lane without a source untouched).
__device__ __forceinline__ uint32_t from_left_lane(uint32_t own_edge, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)own_edge, (int)v, 0x111, 0xf, 0xf, false);   // row_shr:1
}
__device__ __forceinline__ uint32_t from_right_lane(uint32_t own_edge, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)own_edge, (int)v, 0x101, 0xf, 0xf, false);   // row_shl:1
}
template <int PX>
struct Edges { float gl, gr; uint32_t iwe; };   // iwe: idx byte of the left neighbour in bits 7:0, of the right one in 15:8
template <int PX>
__device__ __forceinline__ Edges<PX> edges_of(const Raw<PX>& r, int dr) {
  Edges<PX> e;
  e.gl = __builtin_bit_cast(float, from_left_lane(__builtin_bit_cast(uint32_t, r.ge[dr]), __builtin_bit_cast(uint32_t, r.gc[dr][PX - 1])));
  e.gr = __builtin_bit_cast(float, from_right_lane(__builtin_bit_cast(uint32_t, r.ge[dr]), __builtin_bit_cast(uint32_t, r.gc[dr][0])));
  const uint32_t il = from_left_lane(r.ie[dr], r.ic[dr] >> (8 * (PX - 1)));
  const uint32_t ir = from_right_lane(r.ie[dr], r.ic[dr]);
  e.iwe = (il & 0xffu) | ((ir & 0xffu) << 8);
  return e;
}

// PX = pixels per lane (2 or 4): a wave owns one image row x 16 PX pixels x 64 input channels.  More pixels
// per lane means fewer selects and loads per pixel (the 3 x (PX + 2) neighbourhood is shared by PX pixels).
// LUT: one pool group holds all R orientations of a filter and there is one base bank.  After the max-pool a (filter,
// pixel) carries one orientation, so the gradient reaching BASE tap u' through the neighbour at offset (dy, dx) is
// G * lut[offset][idx][u'] (the rotated banks' coefficients, looked up per value): the routed gradients of all banks
// are summed into the base taps before the contraction, which then runs over the base bank alone, one
// conv-equivalent of matrix work instead of Q, and the neighbourhood is loaded once instead of once per bank.
// RAW: wd is the caller's w[Cout][Cin][9] itself (a plan whose one bank is its base bank, Cin a multiple of 64, Cout of
// 16): a quarter chunk is four filters' 576 contiguous floats of this channel group, loaded 16 bytes per thread as before
// and put into the [tap][channel position] order of the LDS rows by four 4-byte writes at offsets computed once.
template <int PX, bool LUT, int NW, bool RAW = false>
__global__ __launch_bounds__(64 * NW, 2) void k_p4_bwd_data(const float* __restrict__ gpool, const uint8_t* __restrict__ idx,
                                                    const float* __restrict__ wd,
                                                    const int32_t* __restrict__ rot_of, const float* __restrict__ lut,
                                                    float* __restrict__ dx, P4BwdGeom g) {
  constexpr int NT = 64 * NW;
  constexpr int WR = (LUT && NW == 4) ? WROW_TIGHT : WROW;          // LDS floats per filter row
  constexpr int LR = (LUT && NW == 4) ? kLutRowsTight : kLutRows;   // table rows per neighbour offset
  constexpr int WREG = (4 * 9 * (CIG / 4) + NT - 1) / NT;     // staging registers (float4) per quarter chunk and thread
  extern __shared__ float smem[];      // [2][CHUNK][WR], then the tables [base bank][9][LR][12] (LUT)
  float* Tl = smem + 2 * CHUNK * WR;
  if (LUT) {     // a fixed row count per offset: the offset part of a row address is an instruction immediate
    const int R1 = g.R + 1;
    for (int i = threadIdx.x; i < g.Q * 9 * R1 * 12; i += NT) Tl[(i / (R1 * 12)) * (LR * 12) + i % (R1 * 12)] = lut[i];
  }

  const int per_xcd = (g.units + 7) / 8;
  int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (v >= g.units) return;
  // Weight chunks (16 filters of a bank) [c0, c1) of this workgroup: layers with few (row block, strip, channel
  // group) units share their contraction out over ksplit workgroups, each writing an fp32 partial dX that
  // k_p4_sum_dx adds in order.
  const int cpb = g.CoutPad / CHUNK;           // chunks per bank
  const int ksp = v % g.ksplit; v /= g.ksplit;
  const int c0 = ksp * g.kper, c1 = min(g.Q * cpb, c0 + g.kper);
  const int q0 = c0 / cpb, co0 = (c0 % cpb) * CHUNK;      // first K-step: bank, filter
  const int q1 = (c1 - 1) / cpb + 1;                       // banks [q0, q1); the cursors never leave them
  const int cig = v % g.ncig; v /= g.ncig;
  const int strip = v % g.nstrip; v /= g.nstrip;
  const int rb = v % g.nrb;
  const int n = v / g.nrb;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64;
  const int lg = lane / 16, lc = lane % 16;
  const int h = rb * NW + wave;
  const int x0 = strip * 16 * PX;
  const bool active = h < g.H;
  const int HW = g.H * g.W;
  const int nk = (c1 - c0) * (CHUNK / 4);      // K-steps of this workgroup
  const int cbase = c0;                        // its first weight chunk
  const int nchunks = nk / 4;

  // ---- weight chunk streaming -----------------------------------------------------
  // A chunk is 16 filters x 9 taps x 64 channels.  It is copied global -> registers -> LDS a quarter
  // (four filters) per pipeline stage into the buffer the current chunk does not use, so that only two
  // staging registers are live at any time.
  constexpr int Q4 = 4 * 9 * (CIG / 4);        // float4 per quarter chunk (576)
  f4 wreg[WREG];
  // A thread's slots sit at the same byte offsets inside every quarter chunk: computed once, so that a load is a
  // wave-uniform base (chunk, quarter: scalar arithmetic) plus a 32-bit lane offset and costs no vector instruction.
  uint32_t woff[WREG];
  uint32_t wlds[RAW ? WREG : 1][4];      // RAW: LDS byte offsets of a slot's four values inside a quarter's four rows
  const int rowf = g.Cin * 9;            // RAW: floats per filter in w
#pragma unroll
  for (int k = 0; k < WREG; ++k) {
    const int e = min(tid + k * NT, Q4 - 1);
    if (RAW) {
      const int r = e / (9 * (CIG / 4)), j = e % (9 * (CIG / 4));     // filter of the quarter, 16-byte piece of its row
      woff[k] = (uint32_t)((r * rowf + 4 * j) * (int)sizeof(float));
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int m = 4 * j + i, cl = m / 9, u = m % 9;               // channel of the group, tap
        wlds[k][i] = (uint32_t)((r * WR + u * CIG + (cl % 16) * 4 + cl / 16) * (int)sizeof(float));
      }
    } else {
      const int c4 = e % (CIG / 4), u = (e / (CIG / 4)) % 9, r = e / (9 * (CIG / 4));
      woff[k] = (uint32_t)(((r * 9 + u) * g.CinPad + c4 * 4) * (int)sizeof(float));
    }
  }
  const float* wgrp = RAW ? wd + cig * CIG * 9 : wd + cig * CIG;
  auto wload = [&](int cc, int part) {
    const size_t row0 = (size_t)(cbase + cc) * CHUNK + part * 4;      // first filter row of the quarter
    const char* wq = reinterpret_cast<const char*>(wgrp + (RAW ? row0 * rowf : row0 * 9 * g.CinPad));
#pragma unroll
    for (int k = 0; k < WREG; ++k) {
      const int e = tid + k * NT;
      if (e < Q4) wreg[k] = *reinterpret_cast<const f4*>(wq + woff[k]);
    }
  };
  auto wstore = [&](int buf, int part) {
    float* dst = smem + buf * CHUNK * WR;
#pragma unroll
    for (int k = 0; k < WREG; ++k) {
      const int e = tid + k * NT;
      if (e < Q4) {
        if (RAW) {
          char* q4 = reinterpret_cast<char*>(dst + part * 4 * WR);
#pragma unroll
          for (int i = 0; i < 4; ++i) *reinterpret_cast<float*>(q4 + wlds[k][i]) = wreg[k][i];
        } else {
          const int c4 = e % (CIG / 4), u = (e / (CIG / 4)) % 9, r = part * 4 + e / (9 * (CIG / 4));
          *reinterpret_cast<f4*>(dst + r * WR + u * CIG + c4 * 4) = wreg[k];
        }
      }
    }
  };

  // ---- (G, idx) neighbourhood loads -------------------------------------------------------------
  // Everything that depends on the lane only (row / pixel offsets inside a channel plane, validity)
  // is computed once; per K-step the address is a wave-uniform base plus 32-bit lane offsets.
  // Out-of-range positions read a clamped (valid) address and get the idx byte 0xff, which matches no
  // orientation (R <= 255), so they contribute nothing; so do lanes whose filter is beyond Cout (they
  // read the last filter).  Nothing is computed from a loaded value before the K-step that uses it, so the
  // loads stay in flight for two K-steps.
  // A load address is a wave-uniform part -- image, pool group, first filter of the K-step, row (a wave owns one row):
  // scalar arithmetic -- plus a lane part that is the same in every K-step: the lane's filter among the four and its
  // column.  (One image of the pooled gradient has fewer than 2^30 elements: checked when the plan takes this kernel.)
  const int xa = x0 + PX * lc;                 // first of this lane's PX pixels (W % PX == 0: in or out together)
  const uint32_t plane = (uint32_t)g.ng * (uint32_t)HW;          // floats between consecutive filters
  uint32_t rowoff[3], invc[3], inve[3];        // invc: centre bytes, inve: byte 0 left, byte 1 right
#pragma unroll
  for (int dr = 0; dr < 3; ++dr) {
    const int row = h - 1 + dr;
    const bool rok = active && row >= 0 && row < g.H;
    const bool okc = rok && xa < g.W, okl = rok && xa >= 1 && xa - 1 < g.W, okr = rok && xa + PX < g.W;
    rowoff[dr] = (uint32_t)(rok ? row : 0) * (uint32_t)g.W;
    invc[dr] = okc ? 0u : 0xffffffffu;
    inve[dr] = (okl ? 0u : 0xffu) | (okr ? 0u : 0xff00u);
  }
  // the edge load: the row's first lane fetches its left neighbour, the last lane its right neighbour; the lanes
  // between them read the first lane's address too (one cache line for the fifteen; their value is not used)
  const uint32_t colc = (uint32_t)(xa < g.W ? xa : 0);
  const uint32_t cole = lc == 15 ? (uint32_t)(xa + PX < g.W ? xa + PX : 0) : (uint32_t)(x0 >= 1 && x0 - 1 < g.W ? x0 - 1 : 0);
  const uint32_t lgplane = (uint32_t)lg * plane;
  const uint32_t ec = lgplane + colc, ee = lgplane + cole;       // element offsets (the idx bytes), and in bytes of G:
  const uint32_t ec4 = ec * 4u, ee4 = ee * 4u;
  const float* gimg = gpool + (size_t)n * g.Cout * plane;
  const uint8_t* iimg = idx + (size_t)n * g.Cout * plane;
  auto bank_rot = [&](int q, int (&rot)[4]) {                     // orientation index of each quarter turn (-1: absent)
#pragma unroll
    for (int s = 0; s < 4; ++s) rot[s] = rot_of[q * 4 + s];
  };
  auto group_of = [&](const int (&rot)[4]) {                      // pool group the bank's orientations live in
    int r0 = 0;
#pragma unroll
    for (int s = 3; s >= 0; --s) r0 = rot[s] >= 0 ? rot[s] : r0;
    return r0 % g.ng;
  };
  // load cursor: K-step (bank, first filter) that the next raw_load fetches; it stops on the last K-step
  int ld_q = q0, ld_co = co0, ld_pg;
  {
    int r[4];
    bank_rot(q0, r);
    ld_pg = group_of(r);
  }
  auto raw_load = [&](Raw<PX>& r) {
    const int fco = min(ld_co, g.Cout - 1);      // first filter of the K-step (clamped: a K-step of the padding)
    const int lim = g.Cout - 1 - fco;            // lanes with lg > lim hold no filter: they read filter fco + lim
    const size_t kbase = (size_t)ld_pg * HW + (size_t)fco * plane;
    const float* gb = gimg + kbase;
    const uint8_t* ib = iimg + kbase;
    uint32_t oc = ec, oe = ee, oc4 = ec4, oe4 = ee4;
    r.finv = 0u;
    if (lim < 3 || ld_co >= g.Cout) {            // wave-uniform: the K-step reaches beyond Cout
      const uint32_t back = (uint32_t)(lg - min(lg, lim)) * plane;
      oc -= back; oe -= back; oc4 -= back * 4u; oe4 -= back * 4u;
      r.finv = ld_co + lg < g.Cout ? 0u : 0xffffffffu;
    }
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      const char* gr = reinterpret_cast<const char*>(gb + rowoff[dr]);
      const uint8_t* ir = ib + rowoff[dr];
      if (PX == 2) {
        const float2 v = *reinterpret_cast<const float2*>(gr + oc4);
        r.gc[dr][0] = v.x; r.gc[dr][1] = v.y;
        r.ic[dr] = *reinterpret_cast<const uint16_t*>(ir + oc);
      } else {
        const f4 v = *reinterpret_cast<const f4*>(gr + oc4);
#pragma unroll
        for (int p = 0; p < PX; ++p) r.gc[dr][p] = v[p];
        r.ic[dr] = *reinterpret_cast<const uint32_t*>(ir + oc);
      }
      r.ge[dr] = *reinterpret_cast<const float*>(gr + oe4);
      r.ie[dr] = ir[oe];
    }
    if (ld_co + 4 < g.CoutPad) {
      ld_co += 4;
    } else if (ld_q + 1 < q1) {
      ++ld_q;
      ld_co = 0;
      int rr[4];
      bank_rot(ld_q, rr);
      ld_pg = group_of(rr);
    }
  };

  // What the four quarter turns of a K-step share: the neighbour lanes' edge values and the idx words with the bytes of
  // invalid positions forced to 0xff (pinned: formed once per K-step, not once per quarter turn).
  struct Pre { float gl[3], gr[3]; uint32_t iwc[3], iwe[3]; };
  auto prepare = [&](const Raw<PX>& r, Pre& p) {
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      const Edges<PX> e = edges_of(r, dr);
      p.gl[dr] = e.gl; p.gr[dr] = e.gr;
      p.iwc[dr] = r.ic[dr] | invc[dr] | r.finv | (PX == 2 ? 0xffff0000u : 0u);
      p.iwe[dr] = e.iwe | inve[dr] | r.finv;
      asm volatile("" : "+v"(p.gl[dr]), "+v"(p.gr[dr]), "+v"(p.iwc[dr]), "+v"(p.iwe[dr]));
    }
  };
  // One quarter turn's share of the nine tap sums for the lane's pixels (Eq. 12 + the rotated
  // tap positions of Eq. 8): Delta_s on the neighbourhood, added where R_s puts each base tap.
  auto build_slice = [&](const Raw<PX>& r, const Pre& p, int s, int rs, float (&a)[9][PX]) {
    float d[3][PX + 2];
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      d[dr][0] = ((p.iwe[dr] & 0xffu) == (uint32_t)rs) ? p.gl[dr] : 0.f;
      d[dr][PX + 1] = (((p.iwe[dr] >> 8) & 0xffu) == (uint32_t)rs) ? p.gr[dr] : 0.f;
#pragma unroll
      for (int q = 0; q < PX; ++q) d[dr][1 + q] = (((p.iwc[dr] >> (8 * q)) & 0xffu) == (uint32_t)rs) ? r.gc[dr][q] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 9; ++u)
#pragma unroll
      for (int b = 0; b < PX; ++b) {
        const float t = d[2 - tap_i(s, u)][b + 2 - tap_j(s, u)];
        a[u][b] = s == 0 ? t : a[u][b] + t;
      }
  };

  // LUT build of the nine base-tap sums (see the kernel's head).  lut_prepare: per neighbourhood value its gradient
  // (dropped for an idx outside [0, R), which also selects the all-zero table row) and its row offset.  The sums are
  // then formed in 9 PX blocks, block = (row dr, pixel b, column offset dc - 1): nine multiply-adds of the value with
  // the table row of (offset, orientation).  lut_read issues a block's row reads ahead of a tap's matrix instructions,
  // lut_fma consumes them behind those.
  struct LutVals { float gv[3][PX + 2]; uint32_t off[3][PX + 2]; };
  struct LutRow { f4 t0, t1; float t8; };
  auto lut_prepare = [&](const Raw<PX>& r, int bank, LutVals& v) {      // bank: the K-step's base bank (its table)
    const uint32_t tbase = (uint32_t)bank * (9 * LR * 12);
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      const Edges<PX> e = edges_of(r, dr);
      const uint32_t iwc = r.ic[dr] | invc[dr] | r.finv | (PX == 2 ? 0xffff0000u : 0u);
      const uint32_t iwe = e.iwe | inve[dr] | r.finv;
#pragma unroll
      for (int c = 0; c < PX + 2; ++c) {
        const uint32_t byte = c == 0 ? (iwe & 0xffu) : c == PX + 1 ? ((iwe >> 8) & 0xffu) : ((iwc >> (8 * (c - 1))) & 0xffu);
        const float gval = c == 0 ? e.gl : c == PX + 1 ? e.gr : r.gc[dr][c - 1];
        v.gv[dr][c] = byte < (uint32_t)g.R ? gval : 0.f;
        v.off[dr][c] = min(byte, (uint32_t)g.R) * 12u + tbase;
      }
    }
  };
  auto lut_read = [&](const LutVals& v, int blk) -> LutRow {
    const int dr = blk / (3 * PX), bb = (blk % (3 * PX)) / 3, dc = blk % 3;
    const float* t = Tl + (dr * 3 + dc) * (LR * 12) + v.off[dr][bb + dc];   // neighbour at column offset dc - 1 of pixel bb
    LutRow row;
    row.t0 = *reinterpret_cast<const f4*>(t);
    row.t1 = *reinterpret_cast<const f4*>(t + 4);
    row.t8 = t[8];
    return row;
  };
  auto lut_fma = [&](const LutVals& v, int blk, const LutRow& row, float (&a)[9][PX]) {
    const int dr = blk / (3 * PX), bb = (blk % (3 * PX)) / 3, dc = blk % 3;
    const float gvc = v.gv[dr][bb + dc];
    const float tv[9] = {row.t0[0], row.t0[1], row.t0[2], row.t0[3], row.t1[0], row.t1[1], row.t1[2], row.t1[3], row.t8};
#pragma unroll
    for (int u = 0; u < 9; ++u) a[u][bb] = (dr == 0 && dc == 0) ? gvc * tv[u] : a[u][bb] + gvc * tv[u];
  };

  f4 acc[NCB][PX];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int b = 0; b < PX; ++b) acc[cb][b] = f4{0.f, 0.f, 0.f, 0.f};

  // Three-stage pipeline over K-steps: (G, idx) loads two steps ahead, A build one step ahead and
  // spread between the MFMAs of the current step, B reads from LDS one tap ahead.  Scheduling fences
  // keep the loads at the head of the stage; left alone, the compiler sinks them next to their use.
  Raw<PX> rawA, rawB;
  float aA[9][PX], aB[9][PX];
  int rotb[4];                      // orientations of the bank of the K-step being built
  int bd_q = q0, bd_co = co0;       // build cursor
  bank_rot(q0, rotb);
  auto stage = [&](int ks, const float* wl, const Raw<PX>& raw_use, Raw<PX>& raw_ld, const float (&a_cur)[9][PX],
                   float (&a_nxt)[9][PX]) {
    raw_load(raw_ld);
    // the K-step being built is the one after the current one
    if (bd_co + 4 < g.CoutPad) {
      bd_co += 4;
    } else if (bd_q + 1 < q1) {
      ++bd_q;
      bd_co = 0;
      bank_rot(bd_q, rotb);
    }
    __builtin_amdgcn_sched_barrier(0);
    // B operand: one 16-byte LDS read per tap (the lane's channel in the four 16-channel blocks), issued
    // one tap ahead; the fences keep it there.
    f4 bw[2];
    bw[0] = *reinterpret_cast<const f4*>(wl + (ks * 4) * WR);
    // LUT: PX blocks of the next K-step's sums per tap, their table rows read one tap ahead
    LutVals lv;
    LutRow lrow[PX];
    Pre pre;
    if (LUT) lut_prepare(raw_use, bd_q, lv);
    else prepare(raw_use, pre);
#pragma unroll
    for (int u = 0; u < 9; ++u) {
      if (u < 8) bw[(u + 1) & 1] = *reinterpret_cast<const f4*>(wl + (ks * 4) * WR + (u + 1) * CIG);
      if (LUT) {      // read ahead of the tap's matrix instructions, used behind them
#pragma unroll
        for (int i = 0; i < PX; ++i) lrow[i] = lut_read(lv, u * PX + i);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int b = 0; b < PX; ++b)
          acc[cb][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[u][b], bw[u & 1][cb], acc[cb][b], 0, 0, 0);
      if (LUT) {
#pragma unroll
        for (int i = 0; i < PX; ++i) lut_fma(lv, u * PX + i, lrow[i], a_nxt);
        // the sums are first used in the next stage's block: left alone, the compiler sinks all their multiply-adds
        // there and keeps every table row live until then
#pragma unroll
        for (int i = 0; i < PX; ++i)
#pragma unroll
          for (int t = 0; t < 9; ++t) asm volatile("" : "+v"(a_nxt[t][(u * PX + i) % (3 * PX) / 3]));
      } else if ((u & 1) == 0 && u < 8) {
        build_slice(raw_use, pre, u / 2, rotb[u / 2], a_nxt);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  raw_load(rawB);
  if (LUT) __syncthreads();            // the table is in LDS
  if (LUT) {
    LutVals lv;
    lut_prepare(rawB, q0, lv);
#pragma unroll
    for (int blk = 0; blk < 9 * PX; ++blk) {
      lut_fma(lv, blk, lut_read(lv, blk), aA);
      __builtin_amdgcn_sched_barrier(0);      // one block's rows at a time (all at once would spill)
    }
  } else {
    Pre pre;
    prepare(rawB, pre);
#pragma unroll
    for (int s = 0; s < 4; ++s) build_slice(rawB, pre, s, rotb[s], aA);
  }
  raw_load(rawA);
#pragma unroll
  for (int part = 0; part < 4; ++part) {
    wload(0, part);
    wstore(0, part);
  }
  __syncthreads();

  for (int cc = 0; cc < nchunks; ++cc) {
    const bool more = cc + 1 < nchunks;
    const float* wl = smem + (cc & 1) * CHUNK * WR + lg * WR + lc * 4;
    if (more) wload(cc + 1, 0);
    stage(0, wl, rawA, rawB, aA, aB);
    if (more) { wstore((cc + 1) & 1, 0); wload(cc + 1, 1); }
    stage(1, wl, rawB, rawA, aB, aA);
    if (more) { wstore((cc + 1) & 1, 1); wload(cc + 1, 2); }
    stage(2, wl, rawA, rawB, aA, aB);
    if (more) { wstore((cc + 1) & 1, 2); wload(cc + 1, 3); }
    stage(3, wl, rawB, rawA, aB, aA);
    if (more) wstore((cc + 1) & 1, 3);
    __syncthreads();
  }

  // ---- store: lane (lg, lc) holds channel cb*16+lc, pixels x0 + 4*PX*lg + j, j = PX*i + b ----
  if (!active) return;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int ci = cig * CIG + cb * 16 + lc;
    if (ci >= g.Cin) continue;
    const int px = x0 + 4 * PX * lg;
    float* o = dx + (((size_t)ksp * g.N + n) * g.Cin + ci) * HW + (size_t)h * g.W + px;   // ksp > 0 only in the partial buffer
    float vals[4 * PX];
#pragma unroll
    for (int j = 0; j < 4 * PX; ++j) vals[j] = acc[cb][j % PX][j / PX];
    if ((g.W & 3) == 0) {
#pragma unroll
      for (int v4 = 0; v4 < PX; ++v4)
        if (px + 4 * v4 < g.W)
          reinterpret_cast<f4*>(o)[v4] = f4{vals[4 * v4], vals[4 * v4 + 1], vals[4 * v4 + 2], vals[4 * v4 + 3]};
    } else {
#pragma unroll
      for (int j = 0; j < 4 * PX; ++j)
        if (px + j < g.W) o[j] = vals[j];
    }
  }
}

// Layers with more than 64 input channels (one pool group per filter; the table variant or a single bank).  The D of
// a (filter, pixel) does not depend on the input channel, and building it costs as much as the matrix instructions of
// one 64-channel group (table: nine table rows from LDS and 81 multiply-adds; per-bank: 72 selects and 108 adds per
// four pixels), so a workgroup's four waves are NCG channel groups x 4 / NCG rows, and the NCG waves of a row build
// the D of a chunk of 16 filters together: wave cg the K-steps [cg 4/NCG, (cg+1) 4/NCG) of the chunk, every lane the
// operand values of its own (pixels, filter) -- exactly the A-operand layout, so the exchange through LDS is
// [row][K-step][tap][pixel tile][lane], written and read without conflicts.  One buffer, two barriers per chunk of
// 144 PX matrix instructions per wave; two or three workgroups share a CU and fill each other's build phases.  The
// bank is re-laid so that the B operand of (K-step, tap) is one contiguous kilobyte ([group][bank][K-step][tap][lane]
// x four channel blocks) and is read straight from global memory (L2; the waves of a group read the same kilobytes),
// one K-step ahead; (G, idx) of the next chunk are loaded at the head of a chunk's matrix instructions.
template <int PX, bool LUT, int NCG>
__global__ __launch_bounds__(256, 2) void k_p4_bwd_data_shared(const float* __restrict__ gpool,
                                                               const uint8_t* __restrict__ idx,
                                                               const f4* __restrict__ wt,
                                                               const int32_t* __restrict__ rot_of,
                                                               const float* __restrict__ lut,
                                                               float* __restrict__ dx, P4BwdGeom g) {
  constexpr int NT = 256;              // 4 / NCG rows x NCG channel groups
  constexpr int NR = 4 / NCG;          // rows per workgroup
  constexpr int NKS = 4 / NCG;         // K-steps of a chunk that a wave builds
  extern __shared__ float smem[];      // the tables [base bank][9][kLutRows][12] (LUT), then D [NR rows][4][9][PX][64]
  float* Tl = smem;
  typedef float DBuf[4][9][PX][64];    // [K-step][tap][pixel tile][lane]
  DBuf* Dl = reinterpret_cast<DBuf*>(smem + (LUT ? g.Q * 9 * kLutRows * 12 : 0));
  if (LUT) {
    const int R1 = g.R + 1;
    for (int i = threadIdx.x; i < g.Q * 9 * R1 * 12; i += NT) Tl[(i / (R1 * 12)) * (kLutRows * 12) + i % (R1 * 12)] = lut[i];
    __syncthreads();
  }

  const int per_xcd = (g.units + 7) / 8;
  int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (v >= g.units) return;
  const int cpb = g.CoutPad / CHUNK;           // chunks per bank
  const int ksp = v % g.ksplit; v /= g.ksplit;
  const int c0 = ksp * g.kper, c1 = min(g.Q * cpb, c0 + g.kper);
  const int cigw = v % g.ncigw; v /= g.ncigw;
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
  const int x0 = strip * 16 * PX;
  const bool active = h < g.H;
  const int HW = g.H * g.W;

  int rot[4];                                       // per-bank variant: orientation of each quarter turn (-1: absent)
#pragma unroll
  for (int s = 0; s < 4; ++s) rot[s] = LUT ? 0 : rot_of[s];

  // ---- (G, idx) neighbourhood loads (as in the kernel above) ----
  const int xa = x0 + PX * lc;
  uint32_t offc[3], offe[3], invc[3], inve[3];
#pragma unroll
  for (int dr = 0; dr < 3; ++dr) {
    const int row = h - 1 + dr;
    const bool rok = active && row >= 0 && row < g.H;
    const bool okc = rok && xa < g.W, okl = rok && xa >= 1 && xa - 1 < g.W, okr = rok && xa + PX < g.W;
    const uint32_t rowoff = (uint32_t)(rok ? row : 0) * (uint32_t)g.W;
    offc[dr] = rowoff + (uint32_t)(okc ? xa : 0);
    const bool okl0 = rok && x0 >= 1 && x0 - 1 < g.W;
    offe[dr] = lc == 15 ? rowoff + (uint32_t)(okr ? xa + PX : 0) : rowoff + (uint32_t)(okl0 ? x0 - 1 : 0);
    invc[dr] = okc ? 0u : 0xffffffffu;
    inve[dr] = (okl ? 0u : 0xffu) | (okr ? 0u : 0xff00u);
  }
  const float* gimg = gpool + (size_t)n * g.Cout * HW;
  const uint8_t* iimg = idx + (size_t)n * g.Cout * HW;
  auto raw_load = [&](int co, Raw<PX>& r) {      // filter co of the layer (beyond Cout: filter 0, nothing routed)
    const bool fok = co < g.Cout;
    const uint32_t fl = (uint32_t)(fok ? co : 0) * (uint32_t)HW;
    r.finv = fok ? 0u : 0xffffffffu;
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      if (PX == 2) {
        const float2 v2 = *reinterpret_cast<const float2*>(gimg + (fl + offc[dr]));
        r.gc[dr][0] = v2.x; r.gc[dr][1] = v2.y;
        r.ic[dr] = *reinterpret_cast<const uint16_t*>(iimg + (fl + offc[dr]));
      } else {
        const f4 v4 = *reinterpret_cast<const f4*>(gimg + (fl + offc[dr]));
#pragma unroll
        for (int p = 0; p < PX; ++p) r.gc[dr][p] = v4[p & 3];
        r.ic[dr] = *reinterpret_cast<const uint32_t*>(iimg + (fl + offc[dr]));
      }
      r.ge[dr] = gimg[fl + offe[dr]];
      r.ie[dr] = iimg[fl + offe[dr]];
    }
  };
  // per-bank variant: the nine tap sums of the lane's PX pixels (Eq. 12 + the rotated tap positions of Eq. 8)
  auto build_taps = [&](const Raw<PX>& r, float (&a)[9][PX]) {
    float gl[3], gr[3];
    uint32_t iwc[3], iwe[3];
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      const Edges<PX> e = edges_of(r, dr);
      gl[dr] = e.gl; gr[dr] = e.gr;
      iwc[dr] = r.ic[dr] | invc[dr] | r.finv | (PX == 2 ? 0xffff0000u : 0u);
      iwe[dr] = e.iwe | inve[dr] | r.finv;
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const uint32_t rs = (uint32_t)rot[s];
      float d[3][PX + 2];
#pragma unroll
      for (int dr = 0; dr < 3; ++dr) {
        d[dr][0] = ((iwe[dr] & 0xffu) == rs) ? gl[dr] : 0.f;
        d[dr][PX + 1] = (((iwe[dr] >> 8) & 0xffu) == rs) ? gr[dr] : 0.f;
#pragma unroll
        for (int p = 0; p < PX; ++p) d[dr][1 + p] = (((iwc[dr] >> (8 * p)) & 0xffu) == rs) ? r.gc[dr][p] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 9; ++u)
#pragma unroll
        for (int b = 0; b < PX; ++b) {
          const float t = d[2 - tap_i(s, u)][b + 2 - tap_j(s, u)];
          a[u][b] = s == 0 ? t : a[u][b] + t;
        }
    }
  };
  // table variant
  struct LutVals { float gv[3][PX + 2]; uint32_t off[3][PX + 2]; };
  auto lut_prepare = [&](const Raw<PX>& r, int bank, LutVals& lv) {
    const uint32_t tbase = (uint32_t)bank * (9 * kLutRows * 12);
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      const Edges<PX> e = edges_of(r, dr);
      const uint32_t iwc = r.ic[dr] | invc[dr] | r.finv | (PX == 2 ? 0xffff0000u : 0u);
      const uint32_t iwe = e.iwe | inve[dr] | r.finv;
#pragma unroll
      for (int c = 0; c < PX + 2; ++c) {
        const uint32_t byte = c == 0 ? (iwe & 0xffu) : c == PX + 1 ? ((iwe >> 8) & 0xffu) : ((iwc >> (8 * (c - 1))) & 0xffu);
        const float gval = c == 0 ? e.gl : c == PX + 1 ? e.gr : r.gc[dr][c - 1];
        lv.gv[dr][c] = byte < (uint32_t)g.R ? gval : 0.f;
        lv.off[dr][c] = min(byte, (uint32_t)g.R) * 12u + tbase;
      }
    }
  };
  // D of pixel b of the lane's filter, nine base taps: three groups (one per neighbour row) of three table-row reads
  // and 27 multiply-adds, one group's reads in flight at a time
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

  f4 acc[NCB][PX];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int b = 0; b < PX; ++b) acc[cb][b] = f4{0.f, 0.f, 0.f, 0.f};

  // this lane's 16 bytes of B operand of (K-step ks of the workgroup's range, tap u): wl[(ks * 9 + u) * 64]
  const f4* wl = wt + ((size_t)cig * g.Q * cpb + c0) * (4 * 9 * 64) + lane;
  // filter of this lane in K-step ks (0..3) of chunk c
  auto filt = [&](int c, int ks) { return (c % cpb) * CHUNK + 4 * ks + lg; };

  Raw<PX> raw[NKS];
#pragma unroll
  for (int i = 0; i < NKS; ++i) raw_load(filt(c0, cg * NKS + i), raw[i]);
  f4 bw[2][9];
#pragma unroll
  for (int u = 0; u < 9; ++u) bw[0][u] = wl[u * 64];

  for (int c = c0; c < c1; ++c) {
    const int bank = c / cpb;
    // ---- the wave's K-steps of the chunk's D -> LDS ----
#pragma unroll
    for (int i = 0; i < NKS; ++i) {
      if (LUT) {
        LutVals lv;
        lut_prepare(raw[i], bank, lv);
#pragma unroll
        for (int b = 0; b < PX; ++b) {
          float d[9];
          build_pixel(lv, b, d);
#pragma unroll
          for (int u = 0; u < 9; ++u) Dl[rw][cg * NKS + i][u][b][lane] = d[u];
        }
      } else {
        float a[9][PX];
        build_taps(raw[i], a);
#pragma unroll
        for (int u = 0; u < 9; ++u)
#pragma unroll
          for (int b = 0; b < PX; ++b) Dl[rw][cg * NKS + i][u][b][lane] = a[u][b];
      }
    }
    // (G, idx) of the next chunk: in flight during this chunk's matrix instructions (the last chunk reloads itself)
    const int cn = min(c + 1, c1 - 1);
#pragma unroll
    for (int i = 0; i < NKS; ++i) raw_load(filt(cn, cg * NKS + i), raw[i]);
    __syncthreads();
    // ---- the contraction of the chunk: four K-steps of 9 x NCB x PX matrix instructions ----
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      float a[9][PX];
#pragma unroll
      for (int u = 0; u < 9; ++u)
#pragma unroll
        for (int b = 0; b < PX; ++b) a[u][b] = Dl[rw][ks][u][b][lane];
      // B of the next K-step (the workgroup's last one reloads itself)
      const int kn = min((c - c0) * 4 + ks + 1, (c1 - c0) * 4 - 1);
#pragma unroll
      for (int u = 0; u < 9; ++u) bw[(ks + 1) & 1][u] = wl[(size_t)(kn * 9 + u) * 64];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < 9; ++u)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
          for (int b = 0; b < PX; ++b)
            acc[cb][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u][b], bw[ks & 1][u][cb], acc[cb][b], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();          // every wave has read the chunk's D
  }

  // ---- store: lane (lg, lc) holds channel cb*16+lc, pixels x0 + 4 PX lg + j, j = PX i + b ----
  if (!active || !cg_on) return;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int ci = cig * CIG + cb * 16 + lc;
    if (ci >= g.Cin) continue;
    const int px = x0 + 4 * PX * lg;
    float* o = dx + (((size_t)ksp * g.N + n) * g.Cin + ci) * HW + (size_t)h * g.W + px;   // ksp > 0 only in the partial buffer
    float vals[4 * PX];
#pragma unroll
    for (int j = 0; j < 4 * PX; ++j) vals[j] = acc[cb][j % PX][j / PX];
    if ((g.W & 3) == 0) {
#pragma unroll
      for (int v4 = 0; v4 < PX; ++v4)
        if (px + 4 * v4 < g.W)
          reinterpret_cast<f4*>(o)[v4] = f4{vals[4 * v4], vals[4 * v4 + 1], vals[4 * v4 + 2], vals[4 * v4 + 3]};
    } else {
#pragma unroll
      for (int j = 0; j < 4 * PX; ++j)
        if (px + j < g.W) o[j] = vals[j];
    }
  }
}

// base bank(s) -> [channel group of 64][base bank][K-step of 4 filters][tap][lane = (filter, channel)][4 channel blocks]
__global__ __launch_bounds__(256) void k_p4_pack_bwd_shared(const float* __restrict__ w, float* __restrict__ wd, int B,
                                                            int ncig, int CoutPad, int Cin, int Cout) {
  const size_t total = (size_t)ncig * B * CoutPad * 64;     // one thread per (group, bank, filter, channel, block)
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int cb = (int)(e % 4), lc = (int)((e / 4) % 16), lg = (int)((e / 64) % 4);
  size_t r = e / 256;
  const int kstep = (int)(r % (CoutPad / 4)); r /= (CoutPad / 4);
  const int b = (int)(r % B);
  const int cig = (int)(r / B);
  const int co = kstep * 4 + lg, ci = cig * CIG + cb * 16 + lc;
  const bool in = co < Cout && ci < Cin;
  const float* src = w + ((size_t)b * Cout * Cin + (size_t)(in ? co * Cin + ci : 0)) * 9;
  float* dst = wd + ((((size_t)cig * B + b) * (CoutPad / 4) + kstep) * 9 * 64 + lg * 16 + lc) * 4 + cb;
#pragma unroll
  for (int u = 0; u < 9; ++u) dst[(size_t)u * 64 * 4] = in ? src[u] : 0.f;
}

// dx[e] = sum over the bank splits, ascending, of part[s][e] (four elements per thread, scalar tail).
__global__ __launch_bounds__(256) void k_p4_sum_dx(const float* __restrict__ part, float* __restrict__ dx, size_t n_elem,
                                                   int nparts) {
  const size_t n4 = n_elem / 4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
    f4 a = reinterpret_cast<const f4*>(part)[i];
    for (int k = 1; k < nparts; ++k) a += reinterpret_cast<const f4*>(part + (size_t)k * n_elem)[i];
    reinterpret_cast<f4*>(dx)[i] = a;
  }
  for (size_t e = n4 * 4 + (size_t)blockIdx.x * 256 + threadIdx.x; e < n_elem; e += (size_t)gridDim.x * 256) {
    float v = part[e];
    for (int k = 1; k < nparts; ++k) v += part[(size_t)k * n_elem + e];
    dx[e] = v;
  }
}

// base bank(s) -> Q first-quadrant banks laid out [Q][CoutPad][9][CinPad] (zero padded).
__global__ __launch_bounds__(256) void k_p4_pack_bwd(const float* __restrict__ w, float* __restrict__ wd,
                                                     const int32_t* __restrict__ fq_src,
                                                     const float* __restrict__ fq_coef,
                                                     const double* __restrict__ fq_coef64, int Q, int CoutPad,
                                                     int CinPad, int Cin, int Cout, int round16, int base) {
  // base: the base bank itself (Q = 1, no expansion)
  // One thread per (bank, filter, channel position): its nine taps read the same 36 bytes of w.
  const int total = Q * CoutPad * CinPad;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  // Inside each group of 64 channels position p holds channel (p % 4) * 16 + p / 4, so that the four
  // 16-channel blocks of a lane's channel sit side by side (one 16-byte LDS read per tap in the kernel).
  const int pos = e % CinPad;
  const int ci = (pos / CIG) * CIG + (pos % 4) * 16 + (pos % CIG) / 4;
  const int co = (e / CinPad) % CoutPad;
  const int q = e / (CinPad * CoutPad);
  const bool in = co < Cout && ci < Cin;
  const int slices = Cout * Cin;
  const float* src = w + (size_t)(in ? co * Cin + ci : 0) * 9;
  float* dst = wd + ((size_t)(q * CoutPad + co) * 9) * CinPad + pos;
#pragma unroll
  for (int u = 0; u < 9; ++u) {
    float acc = 0.f;
    if (base) {       // q counts the base banks
      acc = in ? src[(size_t)q * slices * 9 + u] : 0.f;
    } else if (round16) {     // bf16 plans: the combination in fp64, rounded to fp32 and to bf16 once each
      double a64 = 0.0;
      for (int z = 0; z < kMaxNnz; ++z) {
        const int s = fq_src[(q * 9 + u) * kMaxNnz + z];
        if (in && s >= 0) a64 += fq_coef64[(q * 9 + u) * kMaxNnz + z] * (double)src[(size_t)(s / 9) * slices * 9 + s % 9];
      }
      acc = bf16_to_f32(f32_to_bf16((float)a64));
    } else {
#pragma unroll
      for (int z = 0; z < kMaxNnz; ++z) {
        const int s = fq_src[(q * 9 + u) * kMaxNnz + z];
        if (in && s >= 0) acc += fq_coef[(q * 9 + u) * kMaxNnz + z] * src[(size_t)(s / 9) * slices * 9 + s % 9];
      }
    }
    dst[(size_t)u * CinPad] = acc;
  }
}

}  // namespace

// The fp32 gradients run over the base bank(s) through the routed-gradient table: one pool group per filter, more
// banks than base banks (plan option bwd_lut = -1 keeps the per-bank kernels).  Decided once, when the plan is created
// (the two variants need different amounts of scratch).
bool p4_bwd_lut_choice(const rotconv_plan* p) {
  if (p->host.lut_bwd.empty() || p->host.Q <= p->B || p->ng != 1 || p->d.R > 32 || p->d.dtype == ROTCONV_BF16) return false;
  if (p->opt.bwd_lut < 0) return false;
  return true;
}
bool p4_bwd_lut(const rotconv_plan* p) { return p->bwd_lut != 0; }
bool p4_bwd_lut16_choice(const rotconv_plan* p) {
  if (p->host.lut_bwd.empty() || p->host.Q <= p->B || p->ng != 1 || p->d.R > 32 || p->d.dtype != ROTCONV_BF16) return false;
  return p->opt.bwd_lut >= 0;
}

bool p4_bwd_data_supported(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  if (d.k != 3 || d.stride != 1 || d.pad != 1) return false;   // bf16 plans run these kernels on widened copies
  if (d.W & 1) return false;
  // the kernels address one image of the pooled gradient with 32-bit byte offsets
  if ((size_t)d.Cout * p->ng * d.H * d.W >= ((size_t)1 << 30)) return false;
  return p4_fwd_pool_mode(p) != kOutUnpooled;  // every bank inside one pool group
}

P4BwdGeom p4_bwd_data_geom(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  P4BwdGeom g{};
  g.N = d.N; g.Cin = d.Cin; g.CinPad = (d.Cin + CIG - 1) / CIG * CIG; g.H = d.H; g.W = d.W; g.Cout = d.Cout;
  g.CoutPad = (d.Cout + 15) / 16 * 16; g.R = d.R; g.Q = p->host.Q; g.ng = p->ng;
  // routed-gradient table instead of per-bank sums
  g.lut = p4_bwd_lut(p) ? 1 : 0;
  if (g.lut) g.Q = p->B;        // the "banks" of the contraction are the base banks
  g.ncig = g.CinPad / CIG;
  // several channel groups, and one pool group per filter with one bank per base bank (the table variant, or a
  // single bank): the groups of a row build D together (k_p4_bwd_data_shared): workgroups of 4 / ncg rows x ncg
  // channel groups
  bool one_bank = !g.lut && g.Q == 1 && g.ng == 1 && p->B == 1;     // ... whose bank is the base bank itself
  for (int u = 0; u < 9 && one_bank; ++u)
    for (int z = 0; z < kMaxNnz; ++z) {
      const int src = p->host.fq_src[u * kMaxNnz + z];
      if (z == 0 ? (src != u || p->host.fq_coef[u * kMaxNnz] != 1.0f) : src >= 0) one_bank = false;
    }
  g.ncg = (g.lut || one_bank) && g.ncig >= 2 ? (g.ncig >= 3 ? 4 : 2) : 1;
  g.ncigw = (g.ncig + g.ncg - 1) / g.ncg;
  // otherwise four-wave workgroups, two per CU; the table variant only with one table of at most 17 rows per offset
  // (two workgroups' weight chunks and tables then fill the 160 KB of LDS exactly)
  g.nw = g.ncg > 1 ? 4 : (g.lut && (p->B != 1 || d.R > 16)) ? 8 : 4;
  const int rows_wg = g.ncg > 1 ? 4 / g.ncg : g.nw;
  g.nrb = (d.H + rows_wg - 1) / rows_wg;
  // pixels per lane: four when the rows are long enough and that still leaves a workgroup per CU
  g.px = ((d.W & 3) == 0 && d.W > 32 && d.N * g.ncig * ((d.H + 7) / 8) * ((d.W + 63) / 64) >= 256) ? 4 : 2;
  // the unshared table build is made for two pixels per lane (four would spill); two groups sharing with four pixels
  // per lane would leave room for one workgroup's D buffer and table per CU only
  if (g.lut && g.ncg <= 2) g.px = 2;
  // sharing workgroups are four waves: four pixels per lane only while that leaves two waves per SIMD
  if (g.ncg > 1 && d.N * g.ncigw * g.nrb * ((d.W + 63) / 64) < 512) g.px = 2;
  g.nstrip = (d.W + 16 * g.px - 1) / (16 * g.px);
  g.units = d.N * g.ncigw * g.nstrip * g.nrb;
  // Few units and a long contraction: share its weight chunks (16 filters of a bank) out so that the chip is filled
  // about twice; at least 8 chunks per workgroup, at most 256 MiB of partial sums.
  const int chunks = g.Q * (g.CoutPad / CHUNK);
  const int full = 256 * 8 / g.nw;      // workgroups that occupy every CU's eight wave slots
  g.ksplit = 1;
  if (g.units < full && chunks >= 16) {
    const double dx_bytes = 4.0 * d.N * d.Cin * d.H * d.W;
    const int want = std::min({chunks / 8, (2 * full + g.units - 1) / g.units, std::max(1, (int)(268435456.0 / dx_bytes))});
    g.kper = (chunks + want - 1) / want;
    g.ksplit = (chunks + g.kper - 1) / g.kper;
  }
  // Still far from filling the chip (small maps): go down to two chunks per workgroup, one when dX is tiny, as long
  // as the partial sums stay within 64 MB.
  if (g.units * g.ksplit < full && chunks >= 2) {
    const double dx_bytes = 4.0 * d.N * d.Cin * d.H * d.W;
    const int want = std::min({chunks / (dx_bytes < 2.0e6 ? 1 : 2), (2 * full + g.units - 1) / g.units,
                               std::max(1, (int)(67108864.0 / dx_bytes))});
    if (want > g.ksplit) {
      g.kper = (chunks + want - 1) / want;
      g.ksplit = (chunks + g.kper - 1) / g.kper;
    }
  }
  if (g.ksplit == 1) g.kper = chunks;
  g.units *= g.ksplit;
  return g;
}

size_t p4_bwd_data_part_floats(const rotconv_plan* p) {
  const P4BwdGeom g = p4_bwd_data_geom(p);
  return g.ksplit > 1 ? (size_t)g.ksplit * p->d.N * p->d.Cin * p->d.H * p->d.W : 0;
}

size_t p4_bwd_data_pack_floats(const rotconv_plan* p) {
  const P4BwdGeom g = p4_bwd_data_geom(p);
  return (size_t)g.Q * g.CoutPad * 9 * g.CinPad;
}

// The input gradient reads the caller's w itself (no packed copy, one dependent launch less): the unshared per-bank
// kernel of a plan whose one bank is its base bank, with whole 64-channel groups and whole 16-filter chunks.
bool p4_bwd_data_raw_weights(const rotconv_plan* p) {
  const P4BwdGeom g = p4_bwd_data_geom(p);
  if (p->d.dtype != ROTCONV_F32 || g.lut || g.ncg > 1 || g.Q != 1 || p->B != 1) return false;
  if (p->d.Cin % CIG || p->d.Cout % CHUNK) return false;
  for (int u = 0; u < 9; ++u)
    for (int z = 0; z < kMaxNnz; ++z) {
      const int src = p->host.fq_src[u * kMaxNnz + z];
      if (z == 0 ? (src != u || p->host.fq_coef[u * kMaxNnz] != 1.0f) : src >= 0) return false;
    }
  return true;
}

void launch_p4_pack_bwd(const rotconv_plan* p, const float* w, float* wd, hipStream_t st) {
  const P4BwdGeom g = p4_bwd_data_geom(p);
  if (g.ncg > 1) {
    const size_t total = (size_t)g.ncig * g.Q * g.CoutPad * 64;
    hipLaunchKernelGGL(k_p4_pack_bwd_shared, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, w, wd, g.Q, g.ncig,
                       g.CoutPad, g.Cin, g.Cout);
    return;
  }
  const int total = g.Q * g.CoutPad * g.CinPad;
  hipLaunchKernelGGL(k_p4_pack_bwd, dim3((total + 255) / 256), dim3(256), 0, st, w, wd, p->dev.fq_src, p->dev.fq_coef,
                     p->dev.fq_coef64,
                     g.Q, g.CoutPad, g.CinPad, g.Cin, g.Cout, p->d.dtype == ROTCONV_BF16 ? 1 : 0, g.lut);
}

void launch_p4_bwd_data(const rotconv_plan* p, const float* gpool, const uint8_t* idx, const float* wd, float* dx_out,
                        float* part, hipStream_t st, bool raw_w) {
  const P4BwdGeom g = p4_bwd_data_geom(p);
  float* dx = g.ksplit > 1 ? part : dx_out;
  if (g.ncg > 1) {
    const size_t lds_s = ((size_t)(g.lut ? g.Q * 9 * kLutRows * 12 : 0) + (size_t)(4 / g.ncg) * 4 * 9 * g.px * 64) * sizeof(float);
    const int grid_s = (g.units + 7) / 8 * 8;
    auto gos = [&](auto kern) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_s);
      hipLaunchKernelGGL(kern, dim3(grid_s), dim3(64 * g.nw), lds_s, st, gpool, idx, reinterpret_cast<const f4*>(wd),
                         p->dev.rot_of, p->dev.lut_bwd, dx, g);
    };
    if (g.lut) {
      if (g.px == 4) { if (g.ncg == 4) gos(k_p4_bwd_data_shared<4, true, 4>); else gos(k_p4_bwd_data_shared<4, true, 2>); }
      else { if (g.ncg == 4) gos(k_p4_bwd_data_shared<2, true, 4>); else gos(k_p4_bwd_data_shared<2, true, 2>); }
    } else {
      if (g.px == 4) { if (g.ncg == 4) gos(k_p4_bwd_data_shared<4, false, 4>); else gos(k_p4_bwd_data_shared<4, false, 2>); }
      else { if (g.ncg == 4) gos(k_p4_bwd_data_shared<2, false, 4>); else gos(k_p4_bwd_data_shared<2, false, 2>); }
    }
    if (g.ksplit > 1) {
      const size_t n_elem = (size_t)p->d.N * p->d.Cin * p->d.H * p->d.W;
      const unsigned blocks = (unsigned)std::max<size_t>(1, std::min<size_t>((n_elem / 4 + 255) / 256, 1u << 16));
      hipLaunchKernelGGL(k_p4_sum_dx, dim3(blocks), dim3(256), 0, st, part, dx_out, n_elem, g.ksplit);
    }
    return;
  }
  const bool tight = g.lut && g.nw == 4;
  const size_t lds = ((size_t)2 * CHUNK * (tight ? WROW_TIGHT : WROW) + (g.lut ? g.Q * 9 * (tight ? kLutRowsTight : kLutRows) * 12 : 0)) * sizeof(float);
  const int grid = (g.units + 7) / 8 * 8;
  auto go = [&](auto kern) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * g.nw), lds, st, gpool, idx, wd, p->dev.rot_of, p->dev.lut_bwd, dx, g);
  };
  const bool raw = raw_w && p4_bwd_data_raw_weights(p);      // wd is the caller's w
  if (g.px == 4) { if (raw) go(k_p4_bwd_data<4, false, 4, true>); else go(k_p4_bwd_data<4, false, 4>); }
  else if (g.lut && g.nw == 4) go(k_p4_bwd_data<2, true, 4>);
  else if (g.lut) go(k_p4_bwd_data<2, true, 8>);
  else if (raw) go(k_p4_bwd_data<2, false, 4, true>);
  else go(k_p4_bwd_data<2, false, 4>);
  if (g.ksplit > 1) {
    const size_t n_elem = (size_t)p->d.N * p->d.Cin * p->d.H * p->d.W;
    const unsigned blocks = (unsigned)std::max<size_t>(1, std::min<size_t>((n_elem / 4 + 255) / 256, 1u << 16));
    hipLaunchKernelGGL(k_p4_sum_dx, dim3(blocks), dim3(256), 0, st, part, dx_out, n_elem, g.ksplit);
  }
}

}  // namespace rotconv
