// Fast weight-gradient kernel for 3x3, stride 1, pad 1 (fp32), fused with the
// orientation max-pool backward (paper Eq. 12, 14, 16 in shared-product form).
//
//   dF_q[co,ci,u] = sum_{n,h,x} D^q_u[co,h,x] * X[ci,h,x]
//   D^q_u[co,h,x] = sum_s Delta_(q,s)[co, h+1-i_s(u), x+1-j_s(u)],   Delta_r = G * 1[idx == r]
//
// Summing the routed gradients of a bank's quarter turns at the rotated tap
// positions BEFORE the contraction is Eq. 16's inverse-rotate-and-accumulate moved
// in front of Eq. 14: one contraction over the pixels per bank instead of four.
// The contraction runs on the fp32 matrix cores with M = 16 filters, N = 16 input
// channels, K = 4 pixels.  A lane owns 8 consecutive pixels of one filter (A role)
// and of one channel (B role) in a 32-pixel strip and walks down the rows of its
// range: every (G, idx) row is loaded and routed per quarter turn once and stays
// in registers for the three rows it serves; D is then built from adds alone, in
// the A-operand layout; X goes straight from global memory into the B operand.
// A wave keeps the 9 x 4 accumulator tiles of its 16 filters x 64 channels (144
// registers) over all its work units; the workgroups' sums ("splits") are added
// afterwards in a fixed order by the reduction kernel, which also applies the
// transposed first-quadrant expansion, so the result is deterministic.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "rotconv_bf16.h"
#include "rotconv_kernels.h"
#include "rotconv_p4.h"

namespace rotconv {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

// NCB (template parameter of both kernels): 16-channel blocks per wave: 4 (64 input channels), or 1 for layers
// with at most 16 input channels (a network's first layer), which would otherwise multiply 48+ padded channels
constexpr int NWAVE = 4;       // waves per workgroup = 16-filter blocks per workgroup
constexpr int NT = 64 * NWAVE;

__device__ __host__ constexpr int tap_i(int s, int u) {
  return s == 0 ? u / 3 : s == 1 ? 2 - u % 3 : s == 2 ? 2 - u / 3 : u % 3;
}
__device__ __host__ constexpr int tap_j(int s, int u) {
  return s == 0 ? u % 3 : s == 1 ? u / 3 : s == 2 ? 2 - u % 3 : 2 - u / 3;
}

struct RowW {            // (G, idx) of one filter on one image row as loaded: the lane's 8 pixels and one neighbour per side
  f4 g0, g1;             // pixels 0..3 and 4..7
  float gl, gr;          // left and right neighbour
  uint32_t i0, i1;       // idx bytes of pixels 0..3 and 4..7
  uint32_t il, ir;       // idx of the neighbours
};

// LUT: one pool group holds all R orientations of a filter and there is one base bank: D is formed for the BASE taps,
// D[u'][pixel] = sum over the 3 x 3 neighbours of G * lut[offset][idx][u'] (idx is one-hot after the max-pool; the
// table row holds the rotated bank's coefficients of the base taps), so the contraction runs once instead of once
// per bank and its result is the base-bank gradient itself.
template <int NCB, bool LUT>
__global__ __launch_bounds__(NT, (NCB == 1 && !LUT) ? 2 : 1) void k_p4_bwd_weight(const float* __restrict__ x, const float* __restrict__ gpool,
                                                      const uint8_t* __restrict__ idx,
                                                      const int32_t* __restrict__ rot_of, const float* __restrict__ lut,
                                                      float* __restrict__ partial, P4BwdWGeom g) {
  constexpr int kLutRows = 33;     // table rows per neighbour offset in LDS (R + 1 <= 33): row addresses = immediate + lane offset
  __shared__ float Tl[LUT ? 2 * 9 * kLutRows * 12 : 4];      // one table per base bank (at most two)
  if (LUT) {
    const int R1 = g.R + 1;
    for (int i = threadIdx.x; i < g.Q * 9 * R1 * 12; i += NT) Tl[(i / (R1 * 12)) * (kLutRows * 12) + i % (R1 * 12)] = lut[i];
    __syncthreads();
  }
  // Consecutive indices go to one XCD: the (bank, filter group, channel group) combinations of one work
  // unit share its X and (G, idx) lines in that XCD's L2, and so do the strips of one row range, whose halo
  // columns lie in their neighbours' lines.
  const int per_xcd = gridDim.x / 8;
  int v = gridDim.x % 8 == 0 ? (blockIdx.x % 8) * per_xcd + blockIdx.x / 8 : blockIdx.x;
  const int cig = v % g.ncig; v /= g.ncig;
  const int fbg = v % g.ncog;                 // group of four (bank, 16-filter block) pairs
  const int split = v / g.ncog;

  const int tid = threadIdx.x;
  const int wave = tid / 64, lane = tid % 64;
  const int lg = lane / 16, lc = lane % 16;
  const int HW = g.H * g.W;
  // The waves of a workgroup take consecutive (bank, 16-filter block) pairs, banks outermost, so that a bank
  // with fewer than 64 filters does not leave waves idle.
  const int nfb = g.CoutPad / 16;                                    // 16-filter blocks per bank
  const int fb_flat = min(fbg * NWAVE + wave, g.Q * nfb - 1);       // an idle wave redoes the last pair
  const bool wave_on = fbg * NWAVE + wave < g.Q * nfb;
  const int q = __builtin_amdgcn_readfirstlane(fb_flat / nfb);   // wave-uniform: keeps the rotation indices scalar
  const int cobase = (fb_flat % nfb) * 16;
  const int co = cobase + lc;                        // this lane's filter (A role)
  const int ci0 = cig * 16 * NCB + lc;               // this lane's channel in block 0 (B role)

  int rot[4];
  int r0 = -1;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    rot[s] = rot_of[q * 4 + s];
    if (r0 < 0 && rot[s] >= 0) r0 = rot[s];
  }
  const bool cok = co < g.Cout && (LUT || r0 >= 0);
  const size_t gplane0 = ((size_t)(cok ? co : 0) * g.ng + (LUT || r0 < 0 ? 0 : r0 % g.ng)) * HW;
  const size_t gimg = (size_t)g.Cout * g.ng * HW;
  const size_t ximg = (size_t)g.Cin * HW;

  // Channel-plane offsets of the lane's NCB channels (clamped; out-of-range channels are masked).
  uint32_t xplane[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int ci = ci0 + cb * 16;
    xplane[cb] = (uint32_t)(ci < g.Cin ? ci : 0) * (uint32_t)HW;
  }

  f4 acc[9][NCB];
#pragma unroll
  for (int u = 0; u < 9; ++u)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[u][cb] = f4{0.f, 0.f, 0.f, 0.f};

  // Routed gradients of one row, per quarter turn: m[s][c] = G where idx == orientation (q, s), else 0
  // (Eq. 12).  Column 0 is the left neighbour, 1..8 the lane's pixels, 9 the right neighbour.  Computed
  // once per row and kept in registers while the row serves as h-1, h and h+1.
  auto select_row = [&](const RowW& r, bool rok, bool pok0, bool pok1, bool lok, bool rok2, float (&m)[4][10]) {
    // positions outside the image (or filters beyond Cout) get the idx byte 0xff, which matches no orientation
    const uint32_t ic0 = (rok && pok0) ? r.i0 : 0xffffffffu, ic1 = (rok && pok1) ? r.i1 : 0xffffffffu;
    const uint32_t il = (rok && lok) ? r.il : 0xffu, ir = (rok && rok2) ? r.ir : 0xffu;
    const float gc[8] = {r.g0[0], r.g0[1], r.g0[2], r.g0[3], r.g1[0], r.g1[1], r.g1[2], r.g1[3]};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const uint32_t rs = (uint32_t)rot[s];   // -1 (absent) matches no byte
      m[s][0] = il == rs ? r.gl : 0.f;
      m[s][9] = ir == rs ? r.gr : 0.f;
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        m[s][1 + p] = ((ic0 >> (8 * p)) & 0xffu) == rs ? gc[p] : 0.f;
        m[s][5 + p] = ((ic1 >> (8 * p)) & 0xffu) == rs ? gc[4 + p] : 0.f;
      }
    }
  };
  // D of pixel t of half j (column 4 j + t + 1 of the rows), all nine taps: each quarter turn's routed
  // gradient is taken where R_s puts the base tap (the tap positions of Eq. 8).  Adds only.
  auto build_pixel = [&](const float (&ma)[4][10], const float (&mb)[4][10], const float (&mc)[4][10], int j, int t,
                         float (&a)[9][4]) {
    auto at = [&](int row, int s, int col) -> float { return row == 0 ? ma[s][col] : row == 1 ? mb[s][col] : mc[s][col]; };
#pragma unroll
    for (int u = 0; u < 9; ++u) {
      float v = at(2 - tap_i(0, u), 0, 4 * j + t + 2 - tap_j(0, u));
#pragma unroll
      for (int s = 1; s < 4; ++s) v += at(2 - tap_i(s, u), s, 4 * j + t + 2 - tap_j(s, u));
      a[u][t] = v;
    }
  };

  // LUT: a row as kept for the three rows it serves: per column (0 left neighbour, 1..8 the lane's pixels, 9 right
  // neighbour) the gradient (zero where the position or its idx is not valid) and the table-row offset of its idx
  // (an idx outside [0, R) selects the all-zero row).
  struct LutRowW { float gv[10]; uint32_t off[10]; };
  auto lut_route = [&](const RowW& r, bool rok, bool pok0, bool pok1, bool lok, bool rok2, LutRowW& m) {
    const uint32_t ic0 = (rok && pok0) ? r.i0 : 0xffffffffu, ic1 = (rok && pok1) ? r.i1 : 0xffffffffu;
    const uint32_t il = (rok && lok) ? r.il : 0xffu, ir = (rok && rok2) ? r.ir : 0xffu;
    const float gc[8] = {r.g0[0], r.g0[1], r.g0[2], r.g0[3], r.g1[0], r.g1[1], r.g1[2], r.g1[3]};
#pragma unroll
    for (int c = 0; c < 10; ++c) {
      const uint32_t byte = c == 0 ? il : c == 9 ? ir : c < 5 ? ((ic0 >> (8 * (c - 1))) & 0xffu) : ((ic1 >> (8 * (c - 5))) & 0xffu);
      const float gval = c == 0 ? r.gl : c == 9 ? r.gr : gc[c - 1];
      m.gv[c] = byte < (uint32_t)g.R ? gval : 0.f;
      m.off[c] = min(byte, (uint32_t)g.R) * 12u + (uint32_t)q * (9 * kLutRows * 12);     // q: the wave's base bank
    }
  };
  struct LutT { f4 t0, t1; float t8; };
  // block (dr, dc) of pixel column pc (1..8): the neighbour in row dr at column pc + dc - 1
  auto lut_read = [&](const LutRowW& row, int dr, int dc, int pc) -> LutT {
    const float* t = Tl + (dr * 3 + dc) * (kLutRows * 12) + row.off[pc + dc - 1];
    LutT v;
    v.t0 = *reinterpret_cast<const f4*>(t);
    v.t1 = *reinterpret_cast<const f4*>(t + 4);
    v.t8 = t[8];
    return v;
  };
  auto lut_fma = [&](const LutRowW& row, int dr, int dc, int pc, const LutT& v, int t, float (&a)[9][4]) {
    const float gvc = row.gv[pc + dc - 1];
    const float tv[9] = {v.t0[0], v.t0[1], v.t0[2], v.t0[3], v.t1[0], v.t1[1], v.t1[2], v.t1[3], v.t8};
#pragma unroll
    for (int u = 0; u < 9; ++u) a[u][t] = (dr == 0 && dc == 0) ? gvc * tv[u] : a[u][t] + gvc * tv[u];
  };

  // Work units: (image, row range, 32-pixel strip).  A lane owns pixels px0 .. px0+7 of the strip; it walks
  // down the rows of the range keeping the (G, idx) rows h-1, h, h+1 in registers (each row of the range is
  // loaded once), X comes straight from global memory into the B operand, a full 128-byte line per channel
  // and row.
  for (int unit = split; unit < g.units; unit += g.splits) {
    int uu = unit;
    const int strip = uu % g.nstrip; uu /= g.nstrip;
    const int rng = uu % g.nrange;
    const int n = uu / g.nrange;
    const int h0 = rng * g.rows_per, h1 = min(g.H, h0 + g.rows_per);
    const int px0 = strip * 32 + 8 * lg;
    const bool pok0 = px0 < g.W, pok1 = px0 + 4 < g.W;       // W % 4 == 0: groups of four are in or out together
    const bool lok = pok0 && px0 >= 1, rok2 = px0 + 8 < g.W;
    const int pc0 = pok0 ? px0 : 0, pc1 = pok1 ? px0 + 4 : 0, pl = lok ? px0 - 1 : 0, pr = rok2 ? px0 + 8 : 0;
    const float* gb = gpool + (size_t)n * gimg + gplane0;
    const uint8_t* ib = idx + (size_t)n * gimg + gplane0;
    const float* xb = x + (size_t)n * ximg;

    // Branch-free loads: out-of-range positions read a safe (clamped) address; what they return is
    // discarded when the row is routed (select_row).  X of pixels beyond the row must be zeroed (D there
    // gathers from in-range neighbours): done where the half is used, and only in a strip that hangs over
    // the row end, so the loads themselves stay unconditional.  Channels beyond Cin land in padded columns
    // of the partial sums that nobody reads.
    const bool tail = strip * 32 + 32 > g.W;       // wave-uniform
    auto mask_x = [&](bool pok, f4 (&b)[NCB]) {
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) b[cb] = pok ? b[cb] : f4{0.f, 0.f, 0.f, 0.f};
    };
    auto row_ok = [&](int h) { return cok && h >= 0 && h < g.H; };
    auto load_row = [&](int h, RowW& r) {
      const uint32_t ro = (uint32_t)min(max(h, 0), g.H - 1) * (uint32_t)g.W;
      r.g0 = *reinterpret_cast<const f4*>(gb + ro + pc0);
      r.g1 = *reinterpret_cast<const f4*>(gb + ro + pc1);
      r.i0 = *reinterpret_cast<const uint32_t*>(ib + ro + pc0);
      r.i1 = *reinterpret_cast<const uint32_t*>(ib + ro + pc1);
      r.gl = gb[ro + pl];
      r.gr = gb[ro + pr];
      r.il = ib[ro + pl];
      r.ir = ib[ro + pr];
    };
    auto route = [&](const RowW& r, int h, float (&m)[4][10]) { select_row(r, row_ok(h), pok0, pok1, lok, rok2, m); };
    auto load_x = [&](int h, int j, f4 (&b)[NCB]) {
      const uint32_t off = (uint32_t)min(h, g.H - 1) * (uint32_t)g.W + (uint32_t)(j == 0 ? pc0 : pc1);
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) b[cb] = *reinterpret_cast<const f4*>(xb + xplane[cb] + off);
    };
    auto mfma_half = [&](const float (&a)[9][4], const f4 (&b)[NCB], int t) {
#pragma unroll
      for (int u = 0; u < 9; ++u)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
          acc[u][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u][t], b[cb][t], acc[u][cb], 0, 0, 0);
    };

    RowW rn;                             // the row being loaded (h + 2)
    float m0[4][10], m1[4][10], m2[4][10];   // routed rows h-1, h, h+1; the roles rotate from row to row
    f4 bA[NCB], bB[NCB];
    float aA[9][4], aB[9][4];
    // One image row: (ma, mb, mc) = rows (h-1, h, h+1).  The D values of the half that comes next are built
    // pixel by pixel between the K-steps of the current half; between the halves the freshly loaded row h+2
    // replaces row h-1.
    auto step = [&](int h, float (&ma)[4][10], float (&mb)[4][10], float (&mc)[4][10]) {
      // The scheduling fences keep the loads where they are issued: half a row (144 MFMAs) ahead of
      // their first use.  Left alone, the compiler sinks each load to its use and waits for it there.
      load_row(h + 2, rn);
      load_x(h, 1, bB);
      __builtin_amdgcn_sched_barrier(0);
      if (tail) mask_x(pok0, bA);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        mfma_half(aA, bA, t);
        build_pixel(ma, mb, mc, 1, t, aB);
      }
      __builtin_amdgcn_sched_barrier(0);
      load_x(h + 1, 0, bA);
      route(rn, h + 2, ma);
      __builtin_amdgcn_sched_barrier(0);
      if (tail) mask_x(pok1, bB);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        mfma_half(aB, bB, t);
        build_pixel(mb, mc, ma, 0, t, aA);
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    // LUT: the same walk with the rows kept as (gradient, table offset) pairs.  Per pixel t of a half: three groups of
    // (three table-row reads, the matrix instructions of three taps, 27 multiply-adds into the next half's D); the
    // fences keep a group's reads ahead of its matrix instructions and the opaque uses keep its multiply-adds behind
    // them (the sums are first needed in the next half: left alone, the compiler sinks all of them there).
    auto lut_half = [&](const float (&a)[9][4], const f4 (&b)[NCB], int t, const LutRowW& ra, const LutRowW& rb,
                        const LutRowW& rc, int j, float (&an)[9][4]) {
      const int pc = 4 * j + t + 1;
#pragma unroll
      for (int dr = 0; dr < 3; ++dr) {
        const LutRowW& row = dr == 0 ? ra : dr == 1 ? rb : rc;
        LutT v[3];
#pragma unroll
        for (int dc = 0; dc < 3; ++dc) v[dc] = lut_read(row, dr, dc, pc);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 3 * dr; u < 3 * dr + 3; ++u)
#pragma unroll
          for (int cb = 0; cb < NCB; ++cb)
            acc[u][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u][t], b[cb][t], acc[u][cb], 0, 0, 0);
#pragma unroll
        for (int dc = 0; dc < 3; ++dc) lut_fma(row, dr, dc, pc, v[dc], t, an);
#pragma unroll
        for (int u = 0; u < 9; ++u) asm volatile("" : "+v"(an[u][t]));
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    LutRowW l0, l1, l2;
    auto lroute = [&](const RowW& r, int h, LutRowW& m) { lut_route(r, row_ok(h), pok0, pok1, lok, rok2, m); };
    auto step_lut = [&](int h, LutRowW& ra, LutRowW& rb, LutRowW& rc) {
      load_row(h + 2, rn);
      load_x(h, 1, bB);
      __builtin_amdgcn_sched_barrier(0);
      if (tail) mask_x(pok0, bA);
#pragma unroll
      for (int t = 0; t < 4; ++t) lut_half(aA, bA, t, ra, rb, rc, 1, aB);
      load_x(h + 1, 0, bA);
      lroute(rn, h + 2, ra);
      __builtin_amdgcn_sched_barrier(0);
      if (tail) mask_x(pok1, bB);
#pragma unroll
      for (int t = 0; t < 4; ++t) lut_half(aB, bB, t, rb, rc, ra, 0, aA);
    };
    if (LUT) {
      load_row(h0 - 1, rn);
      lroute(rn, h0 - 1, l0);
      load_row(h0, rn);
      lroute(rn, h0, l1);
      load_row(h0 + 1, rn);
      lroute(rn, h0 + 1, l2);
      load_x(h0, 0, bA);
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int dr = 0; dr < 3; ++dr)
#pragma unroll
          for (int dc = 0; dc < 3; ++dc) {
            const LutRowW& row = dr == 0 ? l0 : dr == 1 ? l1 : l2;
            lut_fma(row, dr, dc, t + 1, lut_read(row, dr, dc, t + 1), t, aA);
            __builtin_amdgcn_sched_barrier(0);
          }
      for (int h = h0; h < h1; h += 3) {
        step_lut(h, l0, l1, l2);
        if (h + 1 >= h1) break;
        step_lut(h + 1, l1, l2, l0);
        if (h + 2 >= h1) break;
        step_lut(h + 2, l2, l0, l1);
      }
    } else {
      load_row(h0 - 1, rn);
      route(rn, h0 - 1, m0);
      load_row(h0, rn);
      route(rn, h0, m1);
      load_row(h0 + 1, rn);
      route(rn, h0 + 1, m2);
      load_x(h0, 0, bA);
#pragma unroll
      for (int t = 0; t < 4; ++t) build_pixel(m0, m1, m2, 0, t, aA);
      for (int h = h0; h < h1; h += 3) {
        step(h, m0, m1, m2);
        if (h + 1 >= h1) break;
        step(h + 1, m1, m2, m0);
        if (h + 2 >= h1) break;
        step(h + 2, m2, m0, m1);
      }
    }
  }

  // partial[split][q][u][CoutPad][CinPad]; lane holds rows (filters) 4*lg+i, column (channel) lc
  if (wave_on) {
    float* out = partial + ((size_t)(split * g.Q + q) * 9) * g.CoutPad * g.CinPad;
#pragma unroll
    for (int u = 0; u < 9; ++u)
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          out[((size_t)u * g.CoutPad + cobase + 4 * lg + i) * g.CinPad + cig * 16 * NCB + cb * 16 + lc] = acc[u][cb][i];
  }
}

// The table variant for layers with more than 64 input channels.  The D of a filter block does not depend on the
// input channel, and building it (nine table rows from LDS and 81 multiply-adds per pixel and filter) costs about as
// much as the matrix instructions of one 64-channel group, so the NCG waves that take the NCG channel groups of ONE
// filter block build each row's D together -- wave cg the pixels [cg 32/NCG, (cg+1) 32/NCG) of the strip, a lane
// 8/NCG pixels of one filter -- and hand it to each other through LDS ([tap][filter][pixel], fp32, rows of 36 floats;
// a lane reads its eight pixels of a tap with two 16-byte reads).  A workgroup is 4/NCG filter blocks x NCG channel
// groups; one barrier per image row (D of row h + 1 goes into the buffer that row h - 1 was read from before the
// previous barrier), one more between work units.  A row's 288 matrix instructions per wave are spread over the
// 3 * 8/NCG table-read groups of the build of the next row.
template <int NCG>
__global__ __launch_bounds__(NT) void k_p4_bwd_weight_lut_shared(const float* __restrict__ x, const float* __restrict__ gpool,
                                                                 const uint8_t* __restrict__ idx,
                                                                 const float* __restrict__ lut,
                                                                 float* __restrict__ partial, P4BwdWGeom g) {
  constexpr int NCB = 4;
  constexpr int NFB = NWAVE / NCG;     // filter blocks per workgroup
  constexpr int PPL = 8 / NCG;         // pixels of D a lane builds per row
  constexpr int NGRP = 3 * PPL;        // table-read groups per row and lane
  constexpr int kLutRows = 33;         // table rows per neighbour offset in LDS (R + 1 <= 33)
  constexpr int DPITCH = 36;           // floats per (tap, filter) row of D in LDS (32 pixels + padding)
  extern __shared__ float smem_s[];
  float* Tl = smem_s;                                      // [2 * 9 * kLutRows * 12]: one table per base bank (at most two)
  typedef float DBuf[NFB][9][16][DPITCH];                  // [filter block][tap][filter][pixel]
  DBuf* Dl = reinterpret_cast<DBuf*>(smem_s + 2 * 9 * kLutRows * 12);     // two buffers
  {
    const int R1 = g.R + 1;
    for (int i = threadIdx.x; i < g.Q * 9 * R1 * 12; i += NT) Tl[(i / (R1 * 12)) * (kLutRows * 12) + i % (R1 * 12)] = lut[i];
    __syncthreads();
  }
  const int per_xcd = gridDim.x / 8;
  int v = gridDim.x % 8 == 0 ? (blockIdx.x % 8) * per_xcd + blockIdx.x / 8 : blockIdx.x;
  const int cigw = v % g.ncigw; v /= g.ncigw;       // set of NCG channel groups
  const int fbg = v % g.ncog;                       // group of NFB (bank, 16-filter block) pairs
  const int split = v / g.ncog;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64;
  const int lg = lane / 16, lc = lane % 16;
  const int cg = wave % NCG, fbw = wave / NCG;      // the wave's channel group and filter block inside the workgroup
  const int HW = g.H * g.W;
  const int nfb = g.CoutPad / 16;
  const int fb_flat = min(fbg * NFB + fbw, g.Q * nfb - 1);          // idle waves redo the last pair
  const int cig = cigw * NCG + cg;
  const bool wave_on = fbg * NFB + fbw < g.Q * nfb && cig < g.ncig;
  const int q = fb_flat / nfb;                       // the wave's base bank
  const int cobase = (fb_flat % nfb) * 16;
  const int co = cobase + lc;                        // this lane's filter (D builder and A role)
  const int ci0 = cig * 16 * NCB + lc;               // this lane's channel in block 0 (B role)
  const bool cok = co < g.Cout;
  const size_t gplane0 = (size_t)(cok ? co : 0) * HW;          // one pooled plane per filter
  const size_t gimg = (size_t)g.Cout * HW;
  const size_t ximg = (size_t)g.Cin * HW;

  uint32_t xplane[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int ci = ci0 + cb * 16;
    xplane[cb] = (uint32_t)(ci < g.Cin ? ci : 0) * (uint32_t)HW;
  }

  f4 acc[9][NCB];
#pragma unroll
  for (int u = 0; u < 9; ++u)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[u][cb] = f4{0.f, 0.f, 0.f, 0.f};

  // (G, idx) of the lane's PPL build pixels and one neighbour per side on one image row, as loaded; and as kept for
  // the three rows it serves: per column (0 left neighbour, 1..PPL the pixels, PPL + 1 right neighbour) the gradient
  // (zero where the position or its idx is not valid) and the table-row offset of its idx
  struct RowS { float gc[PPL]; float gl, gr; uint32_t iw; uint32_t il, ir; };
  struct LutRowS { float gv[PPL + 2]; uint32_t off[PPL + 2]; };
  auto lut_route = [&](const RowS& r, bool rok, bool pok, bool lok, bool rok2, LutRowS& m) {
    const uint32_t ic = (rok && pok) ? r.iw : 0xffffffffu;
    const uint32_t il = (rok && lok) ? r.il : 0xffu, ir = (rok && rok2) ? r.ir : 0xffu;
#pragma unroll
    for (int c = 0; c < PPL + 2; ++c) {
      const uint32_t byte = c == 0 ? il : c == PPL + 1 ? ir : ((ic >> (8 * (c - 1))) & 0xffu);
      const float gval = c == 0 ? r.gl : c == PPL + 1 ? r.gr : r.gc[c - 1];
      m.gv[c] = byte < (uint32_t)g.R ? gval : 0.f;
      m.off[c] = min(byte, (uint32_t)g.R) * 12u + (uint32_t)q * (9 * kLutRows * 12);
    }
  };
  struct LutT { f4 t0, t1; float t8; };
  auto lut_read = [&](const LutRowS& row, int dr, int dc, int pc) -> LutT {
    const float* t = Tl + (dr * 3 + dc) * (kLutRows * 12) + row.off[pc + dc - 1];
    LutT tv;
    tv.t0 = *reinterpret_cast<const f4*>(t);
    tv.t1 = *reinterpret_cast<const f4*>(t + 4);
    tv.t8 = t[8];
    return tv;
  };
  auto lut_fma = [&](const LutRowS& row, int dr, int dc, int pc, const LutT& tv, float (&d)[9]) {
    const float gvc = row.gv[pc + dc - 1];
    const float t9[9] = {tv.t0[0], tv.t0[1], tv.t0[2], tv.t0[3], tv.t1[0], tv.t1[1], tv.t1[2], tv.t1[3], tv.t8};
#pragma unroll
    for (int u = 0; u < 9; ++u) d[u] = (dr == 0 && dc == 0) ? gvc * t9[u] : d[u] + gvc * t9[u];
  };

  for (int unit = split; unit < g.units; unit += g.splits) {
    int uu = unit;
    const int strip = uu % g.nstrip; uu /= g.nstrip;
    const int rng = uu % g.nrange;
    const int n = uu / g.nrange;
    const int h0 = rng * g.rows_per, h1 = min(g.H, h0 + g.rows_per);
    // builder role: PPL pixels of the wave's share of the strip (W % 4 == 0: in or out of the row together)
    const int bx = cg * (32 / NCG) + lg * PPL;               // first build pixel inside the strip
    const int bx0 = strip * 32 + bx;
    const bool bok = bx0 < g.W;
    const bool lok = bok && bx0 >= 1, rok2 = bx0 + PPL < g.W;
    const int bc = bok ? bx0 : 0, bl = lok ? bx0 - 1 : 0, br = rok2 ? bx0 + PPL : 0;
    // operand role: 8 consecutive pixels of the strip, in two halves
    const int px0 = strip * 32 + 8 * lg;
    const bool pok0 = px0 < g.W, pok1 = px0 + 4 < g.W;
    const int pc0 = pok0 ? px0 : 0, pc1 = pok1 ? px0 + 4 : 0;
    const float* gb = gpool + (size_t)n * gimg + gplane0;
    const uint8_t* ib = idx + (size_t)n * gimg + gplane0;
    const float* xb = x + (size_t)n * ximg;
    const bool tail = strip * 32 + 32 > g.W;       // wave-uniform

    auto row_ok = [&](int h) { return cok && h >= 0 && h < g.H; };
    auto load_row = [&](int h, RowS& r) {
      const uint32_t ro = (uint32_t)min(max(h, 0), g.H - 1) * (uint32_t)g.W;
      if (PPL == 2) {
        const float2 gv2 = *reinterpret_cast<const float2*>(gb + ro + bc);
        r.gc[0] = gv2.x; r.gc[1] = gv2.y;
        r.iw = *reinterpret_cast<const uint16_t*>(ib + ro + bc);
      } else {
        const f4 gv4 = *reinterpret_cast<const f4*>(gb + ro + bc);
#pragma unroll
        for (int i = 0; i < PPL; ++i) r.gc[i] = gv4[i & 3];
        r.iw = *reinterpret_cast<const uint32_t*>(ib + ro + bc);
      }
      r.gl = gb[ro + bl];
      r.gr = gb[ro + br];
      r.il = ib[ro + bl];
      r.ir = ib[ro + br];
    };
    auto lroute = [&](const RowS& r, int h, LutRowS& m) { lut_route(r, row_ok(h), bok, lok, rok2, m); };
    auto load_x = [&](int h, f4 (&b)[2][NCB]) {
      const uint32_t ro = (uint32_t)min(h, g.H - 1) * (uint32_t)g.W;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        b[0][cb] = *reinterpret_cast<const f4*>(xb + xplane[cb] + ro + pc0);
        b[1][cb] = *reinterpret_cast<const f4*>(xb + xplane[cb] + ro + pc1);
      }
    };
    auto build_pixel = [&](const LutRowS& ra, const LutRowS& rb, const LutRowS& rc, int pcol, float (&d)[9],
                           auto&& between) {
#pragma unroll
      for (int dr = 0; dr < 3; ++dr) {
        const LutRowS& row = dr == 0 ? ra : dr == 1 ? rb : rc;
        LutT tv[3];
#pragma unroll
        for (int dc = 0; dc < 3; ++dc) tv[dc] = lut_read(row, dr, dc, pcol);
        __builtin_amdgcn_sched_barrier(0);
        between((pcol - 1) * 3 + dr);
#pragma unroll
        for (int dc = 0; dc < 3; ++dc) lut_fma(row, dr, dc, pcol, tv[dc], d);
#pragma unroll
        for (int u = 0; u < 9; ++u) asm volatile("" : "+v"(d[u]));
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // two neighbouring pixels' D -> LDS
    auto put = [&](int buf, const float (&d0)[9], const float (&d1)[9], int pair) {
#pragma unroll
      for (int u = 0; u < 9; ++u)
        *reinterpret_cast<float2*>(&Dl[buf][fbw][u][lc][bx + 2 * pair]) = make_float2(d0[u], d1[u]);
    };
    // the lane's eight pixels of every tap: a[u][j][t] = D of pixel 4 j + t
    auto get = [&](int buf, f4 (&a)[9][2]) {
#pragma unroll
      for (int u = 0; u < 9; ++u) {
        a[u][0] = *reinterpret_cast<const f4*>(&Dl[buf][fbw][u][lc][8 * lg]);
        a[u][1] = *reinterpret_cast<const f4*>(&Dl[buf][fbw][u][lc][8 * lg + 4]);
      }
    };

    RowS rn;                                          // the row being loaded
    LutRowS l0, l1, l2;                               // routed rows; the roles rotate
    f4 bX[2][NCB], bN[2][NCB];                        // X of row h, and of row h + 1 in flight
    f4 aC[9][2];                                      // D of row h (A operands)
    int par = 0;                                      // buffer that holds D of the current row
    // One image row h: (ra, rb, rc) = routed rows (h, h+1, h+2), aC = D(h).  Row h + 3 and X(h + 1) are loaded ahead;
    // the lane's share of D(h + 1) is built between the matrix instructions of row h and written to the other buffer.
    auto step = [&](int h, LutRowS& ra, LutRowS& rb, LutRowS& rc) {
      load_row(h + 3, rn);
      load_x(h + 1, bN);
      __builtin_amdgcn_sched_barrier(0);
      if (tail) {    // X of pixels beyond the row end must be zero: D there gathers in-range neighbours
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
          bX[0][cb] = pok0 ? bX[0][cb] : f4{0.f, 0.f, 0.f, 0.f};
          bX[1][cb] = pok1 ? bX[1][cb] : f4{0.f, 0.f, 0.f, 0.f};
        }
      }
      // the 8 x 9 x NCB matrix instructions of row h (K-step = pixel t of half j, K = the four lane groups)
      auto mfmas = [&](int grp) {
        constexpr int TOT = 8 * 9 * NCB;
#pragma unroll
        for (int i = grp * TOT / NGRP; i < (grp + 1) * TOT / NGRP; ++i) {
          const int ks = i / (9 * NCB), u = (i / NCB) % 9, cb = i % NCB;
          acc[u][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(aC[u][ks / 4][ks % 4], bX[ks / 4][cb][ks % 4], acc[u][cb], 0, 0, 0);
        }
      };
#pragma unroll
      for (int pr2 = 0; pr2 < PPL / 2; ++pr2) {
        float d0[9], d1[9];
        build_pixel(ra, rb, rc, 2 * pr2 + 1, d0, mfmas);
        build_pixel(ra, rb, rc, 2 * pr2 + 2, d1, mfmas);
        put(par ^ 1, d0, d1, pr2);
        __builtin_amdgcn_sched_barrier(0);
      }
      lroute(rn, h + 3, ra);                          // row h + 3 replaces row h
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) bX[j][cb] = bN[j][cb];
      __syncthreads();
      par ^= 1;
      get(par, aC);
    };
    // prologue: rows h0 - 1, h0, h0 + 1 -> D(h0); then row h0 + 2 takes the place of row h0 - 1
    load_row(h0 - 1, rn);
    lroute(rn, h0 - 1, l0);
    load_row(h0, rn);
    lroute(rn, h0, l1);
    load_row(h0 + 1, rn);
    lroute(rn, h0 + 1, l2);
    load_x(h0, bX);
    __syncthreads();          // every wave is done with the buffers of the previous unit
#pragma unroll
    for (int pr2 = 0; pr2 < PPL / 2; ++pr2) {
      float d0[9], d1[9];
      auto nothing = [](int) {};
      build_pixel(l0, l1, l2, 2 * pr2 + 1, d0, nothing);
      build_pixel(l0, l1, l2, 2 * pr2 + 2, d1, nothing);
      put(0, d0, d1, pr2);
      __builtin_amdgcn_sched_barrier(0);
    }
    load_row(h0 + 2, rn);
    lroute(rn, h0 + 2, l0);
    __syncthreads();
    get(0, aC);
    for (int h = h0; h < h1; h += 3) {
      step(h, l1, l2, l0);
      if (h + 1 >= h1) break;
      step(h + 1, l2, l0, l1);
      if (h + 2 >= h1) break;
      step(h + 2, l0, l1, l2);
    }
  }

  if (wave_on) {
    float* out = partial + ((size_t)(split * g.Q + q) * 9) * g.CoutPad * g.CinPad;
#pragma unroll
    for (int u = 0; u < 9; ++u)
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          out[((size_t)u * g.CoutPad + cobase + 4 * lg + i) * g.CinPad + cig * 16 * NCB + cb * 16 + lc] = acc[u][cb][i];
  }
}

// ---- bfloat16 tensors -------------------------------------------------------------------------------
// Same work decomposition (units, strips, row ranges, splits, one wave = 16 filters x 64 channels, nine
// taps x four channel blocks of accumulators) on v_mfma_f32_16x16x32_bf16: M = 16 filters, N = 16
// channels, K = 32 pixels = the strip, so a lane's 8 consecutive pixels are exactly its K-slice: the X
// row (8 bf16 = one 16-byte load) IS the B operand.  The matrix instruction being 16 times cheaper per
// product than the fp32 one while vector instructions cost the same, the rotated pre-sum D (27 adds per
// pixel on the vector ALU, and a sum that bf16 could not hold exactly) is dropped: each quarter turn's
// routed gradient row m_s = G * 1[idx == (q,s)] (exact bf16 values, Eq. 12) is multiplied on its own,
//     dF_q[co,ci,u] += sum_s  m_s[row h+1-i_s(u)][pixels shifted by 1-j_s(u)] . X[ci][row h]
// four instructions into one accumulator, the shift being a 16-bit funnel shift of the packed row.  The
// result is the exact "bf16 operands, fp32 accumulation" value.  Quarter turns absent from the angle set
// are skipped (wave-uniform).
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));

struct RowB {            // (G, idx) of one filter on one image row as loaded
  u4 g;                  // the lane's 8 pixels (bf16 pairs)
  uint16_t gl, gr;       // left and right neighbour
  uint32_t i0, i1;       // idx bytes of pixels 0..3 and 4..7
  uint8_t il, ir;        // idx of the neighbours
};

template <int NCB>
__global__ __launch_bounds__(NT, NCB == 1 ? 2 : 1) void k_p4_bwd_weight_bf16(const uint16_t* __restrict__ x,
                                                           const uint16_t* __restrict__ gpool,
                                                           const uint8_t* __restrict__ idx,
                                                           const int32_t* __restrict__ rot_of,
                                                           float* __restrict__ partial, P4BwdWGeom g) {
  const int per_xcd = gridDim.x / 8;
  int v = gridDim.x % 8 == 0 ? (blockIdx.x % 8) * per_xcd + blockIdx.x / 8 : blockIdx.x;
  const int cig = v % g.ncig; v /= g.ncig;
  const int fbg = v % g.ncog;
  const int split = v / g.ncog;

  const int tid = threadIdx.x;
  const int wave = tid / 64, lane = tid % 64;
  const int lg = lane / 16, lc = lane % 16;
  const int HW = g.H * g.W;
  const int nfb = g.CoutPad / 16;
  const int fb_flat = min(fbg * NWAVE + wave, g.Q * nfb - 1);       // an idle wave redoes the last pair
  const bool wave_on = fbg * NWAVE + wave < g.Q * nfb;
  const int q = __builtin_amdgcn_readfirstlane(fb_flat / nfb);
  const int cobase = (fb_flat % nfb) * 16;
  const int co = cobase + lc;                        // this lane's filter (A role)
  const int ci0 = cig * 16 * NCB + lc;               // this lane's channel in block 0 (B role)

  int rot[4];
  int r0 = -1;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    rot[s] = __builtin_amdgcn_readfirstlane(rot_of[q * 4 + s]);
    if (r0 < 0 && rot[s] >= 0) r0 = rot[s];
  }
  const bool cok = co < g.Cout && r0 >= 0;
  const size_t gplane0 = ((size_t)(cok ? co : 0) * g.ng + (r0 < 0 ? 0 : r0 % g.ng)) * HW;
  const size_t gimg = (size_t)g.Cout * g.ng * HW;
  const size_t ximg = (size_t)g.Cin * HW;

  uint32_t xplane[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int ci = ci0 + cb * 16;
    xplane[cb] = (uint32_t)(ci < g.Cin ? ci : 0) * (uint32_t)HW;
  }

  f4 acc[9][NCB];
#pragma unroll
  for (int u = 0; u < 9; ++u)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[u][cb] = f4{0.f, 0.f, 0.f, 0.f};

  // Routed row per quarter turn, packed: m[s][0..3] = the lane's 8 pixels (bf16 pairs) with every pixel
  // whose arg-max is not orientation (q, s) zeroed; m[s][4] = right neighbour (low half) and left
  // neighbour (high half), routed the same way.
  auto select_row = [&](const RowB& r, bool rok, bool pok, bool lok, bool rok2, uint32_t (&m)[4][5]) {
    // positions outside the image (or filters beyond Cout) get the idx byte 0xff, which matches no orientation
    const uint32_t iw0 = (rok && pok) ? r.i0 : 0xffffffffu, iw1 = (rok && pok) ? r.i1 : 0xffffffffu;
    const uint32_t il = (rok && lok) ? (uint32_t)r.il : 0xffu, ir = (rok && rok2) ? (uint32_t)r.ir : 0xffu;
    const uint32_t glr = ((uint32_t)r.gl << 16) | (uint32_t)r.gr;
    // the idx bytes of each pixel pair spread to halfwords, then four packed instructions per pair and quarter turn
    const uint32_t x[5] = {__builtin_amdgcn_perm(0u, iw0, 0x0c010c00u), __builtin_amdgcn_perm(0u, iw0, 0x0c030c02u),
                           __builtin_amdgcn_perm(0u, iw1, 0x0c010c00u), __builtin_amdgcn_perm(0u, iw1, 0x0c030c02u),
                           ir | (il << 16)};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const uint32_t rs2 = (uint32_t)rot[s] * 0x00010001u;   // -1 (absent) matches no halfword
#pragma unroll
      for (int j = 0; j < 4; ++j) m[s][j] = r.g[j] & match_mask2(x[j], rs2);
      m[s][4] = glr & match_mask2(x[4], rs2);
    }
  };
  // A operand of (quarter turn s, base tap u): the routed row where R_s puts the tap, its pixels shifted.
  auto operand = [&](const uint32_t (&ma)[4][5], const uint32_t (&mb)[4][5], const uint32_t (&mc)[4][5], int s,
                     int u) -> u4 {
    const int row = 2 - tap_i(s, u), shift = 1 - tap_j(s, u);
    const uint32_t* m = row == 0 ? ma[s] : row == 1 ? mb[s] : mc[s];
    if (shift == 0) return u4{m[0], m[1], m[2], m[3]};
    if (shift < 0)    // pixel t takes pixel t-1: the left neighbour enters from the high half of m[4]
      return u4{__builtin_amdgcn_alignbit(m[0], m[4], 16), __builtin_amdgcn_alignbit(m[1], m[0], 16),
                __builtin_amdgcn_alignbit(m[2], m[1], 16), __builtin_amdgcn_alignbit(m[3], m[2], 16)};
    return u4{__builtin_amdgcn_alignbit(m[1], m[0], 16), __builtin_amdgcn_alignbit(m[2], m[1], 16),
              __builtin_amdgcn_alignbit(m[3], m[2], 16), __builtin_amdgcn_alignbit(m[4], m[3], 16)};
  };

  for (int unit = split; unit < g.units; unit += g.splits) {
    int uu = unit;
    const int strip = uu % g.nstrip; uu /= g.nstrip;
    const int rng = uu % g.nrange;
    const int n = uu / g.nrange;
    const int h0 = rng * g.rows_per, h1 = min(g.H, h0 + g.rows_per);
    const int px0 = strip * 32 + 8 * lg;
    const bool pok = px0 < g.W;                              // W % 8 == 0: a lane's 8 pixels are in or out together
    const bool lok = pok && px0 >= 1, rok2 = px0 + 8 < g.W;
    const int pc = pok ? px0 : 0, pl = lok ? px0 - 1 : 0, pr = rok2 ? px0 + 8 : 0;
    const uint16_t* gb = gpool + (size_t)n * gimg + gplane0;
    const uint8_t* ib = idx + (size_t)n * gimg + gplane0;
    const uint16_t* xb = x + (size_t)n * ximg;
    const bool tail = strip * 32 + 32 > g.W;       // wave-uniform

    auto row_ok = [&](int h) { return cok && h >= 0 && h < g.H; };
    // Branch-free loads: out-of-range positions read a safe (clamped) address; what they return is
    // discarded when the row is routed.
    auto load_row = [&](int h, RowB& r) {
      const uint32_t ro = (uint32_t)min(max(h, 0), g.H - 1) * (uint32_t)g.W;
      r.g = *reinterpret_cast<const u4*>(gb + ro + pc);
      const uint2 iv = *reinterpret_cast<const uint2*>(ib + ro + pc);
      r.i0 = iv.x; r.i1 = iv.y;
      r.gl = gb[ro + pl];
      r.gr = gb[ro + pr];
      r.il = ib[ro + pl];
      r.ir = ib[ro + pr];
    };
    auto route = [&](const RowB& r, int h, uint32_t (&m)[4][5]) { select_row(r, row_ok(h), pok, lok, rok2, m); };
    auto load_x = [&](int h, u4 (&b)[NCB]) {
      const uint32_t off = (uint32_t)min(h, g.H - 1) * (uint32_t)g.W + (uint32_t)pc;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) b[cb] = *reinterpret_cast<const u4*>(xb + xplane[cb] + off);
    };

    RowB rn;                                          // the row being loaded (h + 2)
    uint32_t m0[4][5], m1[4][5], m2[4][5];            // routed rows h-1, h, h+1; the roles rotate
    u4 bX[NCB], bN[NCB];                              // X of row h, and of row h + 1 in flight
    auto step = [&](int h, uint32_t (&ma)[4][5], uint32_t (&mb)[4][5], uint32_t (&mc)[4][5]) {
      // loads a whole row (up to 144 matrix instructions) ahead of their use, fenced so they stay here
      load_row(h + 2, rn);
      load_x(h + 1, bN);
      __builtin_amdgcn_sched_barrier(0);
      if (tail) {    // X of pixels beyond the row end must be zero: the routed rows there gather in-range neighbours
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) bX[cb] = pok ? bX[cb] : u4{0u, 0u, 0u, 0u};
      }
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        if (rot[s] < 0) continue;                     // wave-uniform
#pragma unroll
        for (int u = 0; u < 9; ++u) {
          const bf8 a = __builtin_bit_cast(bf8, operand(ma, mb, mc, s, u));
#pragma unroll
          for (int cb = 0; cb < NCB; ++cb)
            acc[u][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf8, bX[cb]), acc[u][cb], 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      route(rn, h + 2, ma);                           // row h+2 replaces row h-1
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) bX[cb] = bN[cb];
    };
    load_row(h0 - 1, rn);
    route(rn, h0 - 1, m0);
    load_row(h0, rn);
    route(rn, h0, m1);
    load_row(h0 + 1, rn);
    route(rn, h0 + 1, m2);
    load_x(h0, bX);
    for (int h = h0; h < h1; h += 3) {
      step(h, m0, m1, m2);
      if (h + 1 >= h1) break;
      step(h + 1, m1, m2, m0);
      if (h + 2 >= h1) break;
      step(h + 2, m2, m0, m1);
    }
  }

  if (wave_on) {
    float* out = partial + ((size_t)(split * g.Q + q) * 9) * g.CoutPad * g.CinPad;
#pragma unroll
    for (int u = 0; u < 9; ++u)
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          out[((size_t)u * g.CoutPad + cobase + 4 * lg + i) * g.CinPad + cig * 16 * NCB + cb * 16 + lc] = acc[u][cb][i];
  }
}

// bfloat16 tensors, routed-gradient table (one pool group holds all R orientations of a filter, more banks than base
// banks): the gradient that reaches BASE tap u' of a filter at a pixel,
//     D[u'][p] = sum over the 3 x 3 neighbours of G * lut[offset][idx][u'],
// is formed in fp32 from its at most nine terms (vector ALU, table rows from LDS), rounded to bf16 once and used as
// the A operand: ONE matrix instruction per (base tap, channel block) and row instead of one per quarter turn and
// bank (R = 16: 36 instead of 576 per row of 16 filters x 64 channels x 32 pixels), and the result is the base
// bank's gradient itself.  Same units, strips, row ranges and splits as the kernels above.  The D of row h + 1 is
// built, pixel by pixel, between the matrix instructions of row h.
template <int NCB>
__global__ __launch_bounds__(NT, NCB == 1 ? 2 : 1) void k_p4_bwd_weight_bf16_lut(const uint16_t* __restrict__ x,
                                                               const uint16_t* __restrict__ gpool,
                                                               const uint8_t* __restrict__ idx,
                                                               const float* __restrict__ lut,
                                                               float* __restrict__ partial, P4BwdWGeom g) {
  constexpr int kLutRows = 33;     // table rows per neighbour offset in LDS (R + 1 <= 33)
  __shared__ float Tl[2 * 9 * kLutRows * 12];      // one table per base bank (at most two)
  {
    const int R1 = g.R + 1;
    for (int i = threadIdx.x; i < g.Q * 9 * R1 * 12; i += NT) Tl[(i / (R1 * 12)) * (kLutRows * 12) + i % (R1 * 12)] = lut[i];
    __syncthreads();
  }
  const int per_xcd = gridDim.x / 8;
  int v = gridDim.x % 8 == 0 ? (blockIdx.x % 8) * per_xcd + blockIdx.x / 8 : blockIdx.x;
  const int cig = v % g.ncig; v /= g.ncig;
  const int fbg = v % g.ncog;
  const int split = v / g.ncog;

  const int tid = threadIdx.x;
  const int wave = tid / 64, lane = tid % 64;
  const int lg = lane / 16, lc = lane % 16;
  const int HW = g.H * g.W;
  const int nfb = g.CoutPad / 16;
  const int fb_flat = min(fbg * NWAVE + wave, g.Q * nfb - 1);       // an idle wave redoes the last pair
  const bool wave_on = fbg * NWAVE + wave < g.Q * nfb;
  const int q = __builtin_amdgcn_readfirstlane(fb_flat / nfb);      // the wave's base bank
  const int cobase = (fb_flat % nfb) * 16;
  const int co = cobase + lc;                        // this lane's filter (A role)
  const int ci0 = cig * 16 * NCB + lc;               // this lane's channel in block 0 (B role)
  const bool cok = co < g.Cout;
  const size_t gplane0 = (size_t)(cok ? co : 0) * HW;          // one pooled plane per filter
  const size_t gimg = (size_t)g.Cout * HW;
  const size_t ximg = (size_t)g.Cin * HW;

  uint32_t xplane[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int ci = ci0 + cb * 16;
    xplane[cb] = (uint32_t)(ci < g.Cin ? ci : 0) * (uint32_t)HW;
  }

  f4 acc[9][NCB];
#pragma unroll
  for (int u = 0; u < 9; ++u)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[u][cb] = f4{0.f, 0.f, 0.f, 0.f};

  // A row as kept for the three rows it serves: per column (0 left neighbour, 1..8 the lane's pixels, 9 right
  // neighbour) the gradient (zero where the position or its idx is not valid) and the table-row offset of its idx.
  struct LutRowW { float gv[10]; uint32_t off[10]; };
  auto lut_route = [&](const RowB& r, bool rok, bool pok, bool lok, bool rok2, LutRowW& m) {
    const uint32_t ic0 = (rok && pok) ? r.i0 : 0xffffffffu, ic1 = (rok && pok) ? r.i1 : 0xffffffffu;
    const uint32_t il = (rok && lok) ? (uint32_t)r.il : 0xffu, ir = (rok && rok2) ? (uint32_t)r.ir : 0xffu;
#pragma unroll
    for (int c = 0; c < 10; ++c) {
      const uint32_t byte = c == 0 ? il : c == 9 ? ir : c < 5 ? ((ic0 >> (8 * (c - 1))) & 0xffu) : ((ic1 >> (8 * (c - 5))) & 0xffu);
      // bf16 -> fp32: the pair word's low half is the even pixel
      const uint32_t bits = c == 0 ? ((uint32_t)r.gl << 16) : c == 9 ? ((uint32_t)r.gr << 16)
                            : ((c - 1) & 1) ? (r.g[(c - 1) / 2] & 0xffff0000u) : (r.g[(c - 1) / 2] << 16);
      m.gv[c] = byte < (uint32_t)g.R ? __uint_as_float(bits) : 0.f;
      m.off[c] = min(byte, (uint32_t)g.R) * 12u + (uint32_t)q * (9 * kLutRows * 12);
    }
  };
  struct LutT { f4 t0, t1; float t8; };
  auto lut_read = [&](const LutRowW& row, int dr, int dc, int pc) -> LutT {
    const float* t = Tl + (dr * 3 + dc) * (kLutRows * 12) + row.off[pc + dc - 1];
    LutT tv;
    tv.t0 = *reinterpret_cast<const f4*>(t);
    tv.t1 = *reinterpret_cast<const f4*>(t + 4);
    tv.t8 = t[8];
    return tv;
  };
  auto lut_fma = [&](const LutRowW& row, int dr, int dc, int pc, const LutT& tv, float (&d)[9]) {
    const float gvc = row.gv[pc + dc - 1];
    const float t9[9] = {tv.t0[0], tv.t0[1], tv.t0[2], tv.t0[3], tv.t1[0], tv.t1[1], tv.t1[2], tv.t1[3], tv.t8};
#pragma unroll
    for (int u = 0; u < 9; ++u) d[u] = (dr == 0 && dc == 0) ? gvc * t9[u] : d[u] + gvc * t9[u];
  };

  for (int unit = split; unit < g.units; unit += g.splits) {
    int uu = unit;
    const int strip = uu % g.nstrip; uu /= g.nstrip;
    const int rng = uu % g.nrange;
    const int n = uu / g.nrange;
    const int h0 = rng * g.rows_per, h1 = min(g.H, h0 + g.rows_per);
    const int px0 = strip * 32 + 8 * lg;
    const bool pok = px0 < g.W;                              // W % 8 == 0: a lane's 8 pixels are in or out together
    const bool lok = pok && px0 >= 1, rok2 = px0 + 8 < g.W;
    const int pc = pok ? px0 : 0, pl = lok ? px0 - 1 : 0, pr = rok2 ? px0 + 8 : 0;
    const uint16_t* gb = gpool + (size_t)n * gimg + gplane0;
    const uint8_t* ib = idx + (size_t)n * gimg + gplane0;
    const uint16_t* xb = x + (size_t)n * ximg;
    const bool tail = strip * 32 + 32 > g.W;       // wave-uniform

    auto row_ok = [&](int h) { return cok && h >= 0 && h < g.H; };
    auto load_row = [&](int h, RowB& r) {
      const uint32_t ro = (uint32_t)min(max(h, 0), g.H - 1) * (uint32_t)g.W;
      r.g = *reinterpret_cast<const u4*>(gb + ro + pc);
      const uint2 iv = *reinterpret_cast<const uint2*>(ib + ro + pc);
      r.i0 = iv.x; r.i1 = iv.y;
      r.gl = gb[ro + pl];
      r.gr = gb[ro + pr];
      r.il = ib[ro + pl];
      r.ir = ib[ro + pr];
    };
    auto lroute = [&](const RowB& r, int h, LutRowW& m) { lut_route(r, row_ok(h), pok, lok, rok2, m); };
    auto load_x = [&](int h, u4 (&b)[NCB]) {
      const uint32_t off = (uint32_t)min(h, g.H - 1) * (uint32_t)g.W + (uint32_t)pc;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) b[cb] = *reinterpret_cast<const u4*>(xb + xplane[cb] + off);
    };
    // D of pixel column pcol (1..8) from the rows (above, at, below), nine base taps: three groups (one per row) of
    // three table-row reads and 27 multiply-adds.  `between(group)` is issued between a group's reads and its
    // multiply-adds (the matrix instructions of the current row go there); the fences keep the reads of one group
    // at a time in flight and the opaque uses keep the multiply-adds where they are written (the sums are first
    // needed when the row is packed: left alone the compiler gathers all table reads of a row up front).
    auto build_pixel = [&](const LutRowW& ra, const LutRowW& rb, const LutRowW& rc, int pcol, float (&d)[9],
                           auto&& between) {
#pragma unroll
      for (int dr = 0; dr < 3; ++dr) {
        const LutRowW& row = dr == 0 ? ra : dr == 1 ? rb : rc;
        LutT tv[3];
#pragma unroll
        for (int dc = 0; dc < 3; ++dc) tv[dc] = lut_read(row, dr, dc, pcol);
        __builtin_amdgcn_sched_barrier(0);
        between((pcol - 1) * 3 + dr);
#pragma unroll
        for (int dc = 0; dc < 3; ++dc) lut_fma(row, dr, dc, pcol, tv[dc], d);
#pragma unroll
        for (int u = 0; u < 9; ++u) asm volatile("" : "+v"(d[u]));
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    auto pack = [&](const float (&d0)[9], const float (&d1)[9], int pair, u4 (&a)[9]) {
#pragma unroll
      for (int u = 0; u < 9; ++u) {
        typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
        bf2 pr2;
        pr2[0] = (__bf16)d0[u];
        pr2[1] = (__bf16)d1[u];
        a[u][pair] = __builtin_bit_cast(uint32_t, pr2);
      }
    };

    RowB rn;                                          // the row being loaded
    LutRowW l0, l1, l2;                               // routed rows; the roles rotate
    u4 bX[NCB], bN[NCB];                              // X of row h, and of row h + 1 in flight
    u4 aC[9], aN[9];                                  // D of row h (A operands), and of row h + 1 being built
    // One image row h: (ra, rb, rc) = routed rows (h, h+1, h+2), aC = D(h).  Row h + 3 and X(h + 1) are loaded ahead;
    // the D of row h + 1 is built two pixels at a time between the matrix instructions of row h.
    auto step = [&](int h, LutRowW& ra, LutRowW& rb, LutRowW& rc) {
      load_row(h + 3, rn);
      load_x(h + 1, bN);
      __builtin_amdgcn_sched_barrier(0);
      if (tail) {    // X of pixels beyond the row end must be zero: D there gathers in-range neighbours
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) bX[cb] = pok ? bX[cb] : u4{0u, 0u, 0u, 0u};
      }
      // the 9 NCB matrix instructions of row h, spread over the 24 groups of the D build of row h + 1
      auto mfmas = [&](int grp) {
        constexpr int TOT = 9 * NCB;
#pragma unroll
        for (int i = grp * TOT / 24; i < (grp + 1) * TOT / 24; ++i)
          acc[i / NCB][i % NCB] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, aC[i / NCB]),
                                                                          __builtin_bit_cast(bf8, bX[i % NCB]),
                                                                          acc[i / NCB][i % NCB], 0, 0, 0);
      };
#pragma unroll
      for (int pr2 = 0; pr2 < 4; ++pr2) {
        float d0[9], d1[9];
        build_pixel(ra, rb, rc, 2 * pr2 + 1, d0, mfmas);
        build_pixel(ra, rb, rc, 2 * pr2 + 2, d1, mfmas);
        pack(d0, d1, pr2, aN);
        __builtin_amdgcn_sched_barrier(0);
      }
      lroute(rn, h + 3, ra);                          // row h + 3 replaces row h
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) bX[cb] = bN[cb];
#pragma unroll
      for (int u = 0; u < 9; ++u) aC[u] = aN[u];
    };
    // prologue: rows h0 - 1, h0, h0 + 1 -> D(h0); then row h0 + 2 takes the place of row h0 - 1
    load_row(h0 - 1, rn);
    lroute(rn, h0 - 1, l0);
    load_row(h0, rn);
    lroute(rn, h0, l1);
    load_row(h0 + 1, rn);
    lroute(rn, h0 + 1, l2);
    load_x(h0, bX);
#pragma unroll
    for (int pr2 = 0; pr2 < 4; ++pr2) {
      float d0[9], d1[9];
      auto nothing = [](int) {};
      build_pixel(l0, l1, l2, 2 * pr2 + 1, d0, nothing);
      build_pixel(l0, l1, l2, 2 * pr2 + 2, d1, nothing);
      pack(d0, d1, pr2, aC);
      __builtin_amdgcn_sched_barrier(0);
    }
    load_row(h0 + 2, rn);
    lroute(rn, h0 + 2, l0);
    // step(h, rows h, h+1, h+2): the D of row h + 1 is built from exactly those rows
    for (int h = h0; h < h1; h += 3) {
      step(h, l1, l2, l0);
      if (h + 1 >= h1) break;
      step(h + 1, l2, l0, l1);
      if (h + 2 >= h1) break;
      step(h + 2, l0, l1, l2);
    }
  }

  if (wave_on) {
    float* out = partial + ((size_t)(split * g.Q + q) * 9) * g.CoutPad * g.CinPad;
#pragma unroll
    for (int u = 0; u < 9; ++u)
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          out[((size_t)u * g.CoutPad + cobase + 4 * lg + i) * g.CinPad + cig * 16 * NCB + cb * 16 + lc] = acc[u][cb][i];
  }
}

// The same kernel for layers with more than 64 input channels: the D of a filter block does not depend on the input
// channel, and building it (nine table rows from LDS per pixel and filter) is what bounds the kernel above, so the
// NCG waves that take the NCG channel groups of ONE filter block build each row's D together -- wave cg the pixels
// [cg 32/NCG, (cg+1) 32/NCG) of the strip, a lane 8/NCG pixels of one filter -- and hand it to each other through
// LDS as packed bf16 pairs in the A-operand layout ([tap][filter][pixel pair], one 16-byte read per tap and lane).
// A workgroup is 4/NCG filter blocks x NCG channel groups; one barrier per image row (D of row h + 1 is written into
// the buffer that row h - 1 was read from before the previous barrier), one more between work units.
template <int NCB, int NCG, int NW>
__global__ __launch_bounds__(64 * NW) void k_p4_bwd_weight_bf16_lut_shared(const uint16_t* __restrict__ x,
                                                                      const uint16_t* __restrict__ gpool,
                                                                      const uint8_t* __restrict__ idx,
                                                                      const float* __restrict__ lut,
                                                                      float* __restrict__ partial, P4BwdWGeom g) {
  constexpr int NTW = 64 * NW;         // threads per workgroup
  constexpr int NFB = NW / NCG;        // filter blocks per workgroup
  constexpr int PPL = 8 / NCG;         // pixels of D a lane builds per row
  constexpr int NGRP = 3 * PPL;        // table-read groups per row and lane
  constexpr int kLutRows = 33;         // table rows per neighbour offset in LDS (R + 1 <= 33)
  extern __shared__ float smem_w[];
  float* Tl = smem_w;                                      // [2 * 9 * kLutRows * 12]: one table per base bank (at most two)
  typedef uint32_t DBuf[NFB][9][16][16];                   // [filter block][tap][filter][pixel pair]
  DBuf* Dl = reinterpret_cast<DBuf*>(smem_w + 2 * 9 * kLutRows * 12);     // two buffers
  {
    const int R1 = g.R + 1;
    for (int i = threadIdx.x; i < g.Q * 9 * R1 * 12; i += NTW) Tl[(i / (R1 * 12)) * (kLutRows * 12) + i % (R1 * 12)] = lut[i];
    __syncthreads();
  }
  const int per_xcd = gridDim.x / 8;
  int v = gridDim.x % 8 == 0 ? (blockIdx.x % 8) * per_xcd + blockIdx.x / 8 : blockIdx.x;
  const int cigw = v % g.ncigw; v /= g.ncigw;       // group of NCG channel groups
  const int fbg = v % g.ncog;                       // group of NFB (bank, 16-filter block) pairs
  const int split = v / g.ncog;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64;
  const int lg = lane / 16, lc = lane % 16;
  const int cg = wave % NCG, fbw = wave / NCG;      // the wave's channel group and filter block inside the workgroup
  const int HW = g.H * g.W;
  const int nfb = g.CoutPad / 16;
  const int fb_flat = min(fbg * NFB + fbw, g.Q * nfb - 1);          // idle waves redo the last pair
  const int cig = cigw * NCG + cg;
  const bool wave_on = fbg * NFB + fbw < g.Q * nfb && cig < g.ncig;
  const int q = fb_flat / nfb;                       // the wave's base bank
  const int cobase = (fb_flat % nfb) * 16;
  const int co = cobase + lc;                        // this lane's filter (D builder and A role)
  const int ci0 = cig * 16 * NCB + lc;               // this lane's channel in block 0 (B role)
  const bool cok = co < g.Cout;
  const size_t gplane0 = (size_t)(cok ? co : 0) * HW;          // one pooled plane per filter
  const size_t gimg = (size_t)g.Cout * HW;
  const size_t ximg = (size_t)g.Cin * HW;

  uint32_t xplane[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int ci = ci0 + cb * 16;
    xplane[cb] = (uint32_t)(ci < g.Cin ? ci : 0) * (uint32_t)HW;
  }

  f4 acc[9][NCB];
#pragma unroll
  for (int u = 0; u < 9; ++u)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[u][cb] = f4{0.f, 0.f, 0.f, 0.f};

  // (G, idx) of the lane's PPL build pixels and one neighbour per side on one image row, as loaded; and as kept for
  // the three rows it serves: per column (0 left neighbour, 1..PPL the pixels, PPL + 1 right neighbour) the gradient
  // (zero where the position or its idx is not valid) and the table-row offset of its idx
  struct RowS { uint32_t gw[PPL / 2]; uint16_t gl, gr; uint32_t iw; uint8_t il, ir; };
  struct LutRowS { float gv[PPL + 2]; uint32_t off[PPL + 2]; };
  auto lut_route = [&](const RowS& r, bool rok, bool pok, bool lok, bool rok2, LutRowS& m) {
    const uint32_t ic = (rok && pok) ? r.iw : 0xffffffffu;
    const uint32_t il = (rok && lok) ? (uint32_t)r.il : 0xffu, ir = (rok && rok2) ? (uint32_t)r.ir : 0xffu;
#pragma unroll
    for (int c = 0; c < PPL + 2; ++c) {
      const uint32_t byte = c == 0 ? il : c == PPL + 1 ? ir : ((ic >> (8 * (c - 1))) & 0xffu);
      // bf16 -> fp32: the pair word's low half is the even pixel
      const uint32_t bits = c == 0 ? ((uint32_t)r.gl << 16) : c == PPL + 1 ? ((uint32_t)r.gr << 16)
                            : ((c - 1) & 1) ? (r.gw[(c - 1) / 2] & 0xffff0000u) : (r.gw[(c - 1) / 2] << 16);
      m.gv[c] = byte < (uint32_t)g.R ? __uint_as_float(bits) : 0.f;
      m.off[c] = min(byte, (uint32_t)g.R) * 12u + (uint32_t)q * (9 * kLutRows * 12);
    }
  };
  struct LutT { f4 t0, t1; float t8; };
  auto lut_read = [&](const LutRowS& row, int dr, int dc, int pc) -> LutT {
    const float* t = Tl + (dr * 3 + dc) * (kLutRows * 12) + row.off[pc + dc - 1];
    LutT tv;
    tv.t0 = *reinterpret_cast<const f4*>(t);
    tv.t1 = *reinterpret_cast<const f4*>(t + 4);
    tv.t8 = t[8];
    return tv;
  };
  auto lut_fma = [&](const LutRowS& row, int dr, int dc, int pc, const LutT& tv, float (&d)[9]) {
    const float gvc = row.gv[pc + dc - 1];
    const float t9[9] = {tv.t0[0], tv.t0[1], tv.t0[2], tv.t0[3], tv.t1[0], tv.t1[1], tv.t1[2], tv.t1[3], tv.t8};
#pragma unroll
    for (int u = 0; u < 9; ++u) d[u] = (dr == 0 && dc == 0) ? gvc * t9[u] : d[u] + gvc * t9[u];
  };

  for (int unit = split; unit < g.units; unit += g.splits) {
    int uu = unit;
    const int strip = uu % g.nstrip; uu /= g.nstrip;
    const int rng = uu % g.nrange;
    const int n = uu / g.nrange;
    const int h0 = rng * g.rows_per, h1 = min(g.H, h0 + g.rows_per);
    // builder role: PPL pixels of the wave's share of the strip
    const int bpair = cg * (16 / NCG) + lg * (PPL / 2);      // first pixel pair of the lane inside the strip
    const int bx0 = strip * 32 + 2 * bpair;
    const bool bok = bx0 < g.W;                               // W % 8 == 0: the lane's pixels are in or out together
    const bool lok = bok && bx0 >= 1, rok2 = bx0 + PPL < g.W;
    const int bc = bok ? bx0 : 0, bl = lok ? bx0 - 1 : 0, br = rok2 ? bx0 + PPL : 0;
    // operand role: 8 consecutive pixels of the strip
    const int px0 = strip * 32 + 8 * lg;
    const bool pok = px0 < g.W;
    const int pc = pok ? px0 : 0;
    const uint16_t* gb = gpool + (size_t)n * gimg + gplane0;
    const uint8_t* ib = idx + (size_t)n * gimg + gplane0;
    const uint16_t* xb = x + (size_t)n * ximg;
    const bool tail = strip * 32 + 32 > g.W;       // wave-uniform

    auto row_ok = [&](int h) { return cok && h >= 0 && h < g.H; };
    auto load_row = [&](int h, RowS& r) {
      const uint32_t ro = (uint32_t)min(max(h, 0), g.H - 1) * (uint32_t)g.W;
      if (PPL == 2) {
        r.gw[0] = *reinterpret_cast<const uint32_t*>(gb + ro + bc);
        r.iw = *reinterpret_cast<const uint16_t*>(ib + ro + bc);
      } else {
        const uint2 gv2 = *reinterpret_cast<const uint2*>(gb + ro + bc);
        r.gw[0] = gv2.x; r.gw[PPL / 2 - 1] = gv2.y;
        r.iw = *reinterpret_cast<const uint32_t*>(ib + ro + bc);
      }
      r.gl = gb[ro + bl];
      r.gr = gb[ro + br];
      r.il = ib[ro + bl];
      r.ir = ib[ro + br];
    };
    auto lroute = [&](const RowS& r, int h, LutRowS& m) { lut_route(r, row_ok(h), bok, lok, rok2, m); };
    auto load_x = [&](int h, u4 (&b)[NCB]) {
      const uint32_t off = (uint32_t)min(h, g.H - 1) * (uint32_t)g.W + (uint32_t)pc;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) b[cb] = *reinterpret_cast<const u4*>(xb + xplane[cb] + off);
    };
    // D of pixel column pcol (1..PPL) from the rows (above, at, below): three groups (one per row) of three table-row
    // reads and 27 multiply-adds, `between(group)` issued between a group's reads and its multiply-adds; fences and
    // opaque uses as in the kernel above
    auto build_pixel = [&](const LutRowS& ra, const LutRowS& rb, const LutRowS& rc, int pcol, float (&d)[9],
                           auto&& between) {
#pragma unroll
      for (int dr = 0; dr < 3; ++dr) {
        const LutRowS& row = dr == 0 ? ra : dr == 1 ? rb : rc;
        LutT tv[3];
#pragma unroll
        for (int dc = 0; dc < 3; ++dc) tv[dc] = lut_read(row, dr, dc, pcol);
        __builtin_amdgcn_sched_barrier(0);
        between((pcol - 1) * 3 + dr);
#pragma unroll
        for (int dc = 0; dc < 3; ++dc) lut_fma(row, dr, dc, pcol, tv[dc], d);
#pragma unroll
        for (int u = 0; u < 9; ++u) asm volatile("" : "+v"(d[u]));
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // a pixel pair's D -> LDS (bf16 pairs), A-operand layout
    auto put = [&](int buf, const float (&d0)[9], const float (&d1)[9], int pair) {
#pragma unroll
      for (int u = 0; u < 9; ++u) {
        typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
        bf2 pr2;
        pr2[0] = (__bf16)d0[u];
        pr2[1] = (__bf16)d1[u];
        Dl[buf][fbw][u][lc][bpair + pair] = __builtin_bit_cast(uint32_t, pr2);
      }
    };
    auto get = [&](int buf, u4 (&a)[9]) {
#pragma unroll
      for (int u = 0; u < 9; ++u) a[u] = *reinterpret_cast<const u4*>(&Dl[buf][fbw][u][lc][4 * lg]);
    };

    RowS rn;                                          // the row being loaded
    LutRowS l0, l1, l2;                               // routed rows; the roles rotate
    u4 bX[NCB], bN[NCB];                              // X of row h, and of row h + 1 in flight
    u4 aC[9];                                         // D of row h (A operands)
    int par = 0;                                      // buffer that holds D of the current row
    // One image row h: (ra, rb, rc) = routed rows (h, h+1, h+2), aC = D(h).  Row h + 3 and X(h + 1) are loaded ahead;
    // the lane's share of D(h + 1) is built between the matrix instructions of row h and written to the other buffer.
    auto step = [&](int h, LutRowS& ra, LutRowS& rb, LutRowS& rc) {
      load_row(h + 3, rn);
      load_x(h + 1, bN);
      __builtin_amdgcn_sched_barrier(0);
      if (tail) {    // X of pixels beyond the row end must be zero: D there gathers in-range neighbours
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) bX[cb] = pok ? bX[cb] : u4{0u, 0u, 0u, 0u};
      }
      auto mfmas = [&](int grp) {
        constexpr int TOT = 9 * NCB;
#pragma unroll
        for (int i = grp * TOT / NGRP; i < (grp + 1) * TOT / NGRP; ++i)
          acc[i / NCB][i % NCB] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, aC[i / NCB]),
                                                                          __builtin_bit_cast(bf8, bX[i % NCB]),
                                                                          acc[i / NCB][i % NCB], 0, 0, 0);
      };
#pragma unroll
      for (int pr2 = 0; pr2 < PPL / 2; ++pr2) {
        float d0[9], d1[9];
        build_pixel(ra, rb, rc, 2 * pr2 + 1, d0, mfmas);
        build_pixel(ra, rb, rc, 2 * pr2 + 2, d1, mfmas);
        put(par ^ 1, d0, d1, pr2);
        __builtin_amdgcn_sched_barrier(0);
      }
      lroute(rn, h + 3, ra);                          // row h + 3 replaces row h
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) bX[cb] = bN[cb];
      __syncthreads();
      par ^= 1;
      get(par, aC);
    };
    // prologue: rows h0 - 1, h0, h0 + 1 -> D(h0); then row h0 + 2 takes the place of row h0 - 1
    load_row(h0 - 1, rn);
    lroute(rn, h0 - 1, l0);
    load_row(h0, rn);
    lroute(rn, h0, l1);
    load_row(h0 + 1, rn);
    lroute(rn, h0 + 1, l2);
    load_x(h0, bX);
    __syncthreads();          // every wave is done with the buffers of the previous unit
#pragma unroll
    for (int pr2 = 0; pr2 < PPL / 2; ++pr2) {
      float d0[9], d1[9];
      auto nothing = [](int) {};
      build_pixel(l0, l1, l2, 2 * pr2 + 1, d0, nothing);
      build_pixel(l0, l1, l2, 2 * pr2 + 2, d1, nothing);
      put(0, d0, d1, pr2);
      __builtin_amdgcn_sched_barrier(0);
    }
    load_row(h0 + 2, rn);
    lroute(rn, h0 + 2, l0);
    __syncthreads();
    get(0, aC);
    for (int h = h0; h < h1; h += 3) {
      step(h, l1, l2, l0);
      if (h + 1 >= h1) break;
      step(h + 1, l2, l0, l1);
      if (h + 2 >= h1) break;
      step(h + 2, l0, l1, l2);
    }
  }

  if (wave_on) {
    float* out = partial + ((size_t)(split * g.Q + q) * 9) * g.CoutPad * g.CinPad;
#pragma unroll
    for (int u = 0; u < 9; ++u)
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          out[((size_t)u * g.CoutPad + cobase + 4 * lg + i) * g.CinPad + cig * 16 * NCB + cb * 16 + lc] = acc[u][cb][i];
  }
}

// Where the summed dF goes.  RELAYOUT: the transposed expansion is the identity (the table variant, whose dF already is
// the base banks' gradient, or a plan whose one bank is its base bank): element ((b*9 + u) * CoutPad + co) * CinPad + ci of
// dF is dw[b][co][ci][u], written directly -- one launch instead of two, the same sums in the same order.
struct DwLayout { int Cout, Cin, CoutPad, CinPad; };
template <bool RELAYOUT>
__device__ __forceinline__ void put_sum(float* __restrict__ out, int e, float v, const DwLayout& L) {
  if (!RELAYOUT) { out[e] = v; return; }
  const int ci = e % L.CinPad, co = (e / L.CinPad) % L.CoutPad, bu = e / (L.CinPad * L.CoutPad);
  if (ci < L.Cin && co < L.Cout) out[(((size_t)(bu / 9) * L.Cout + co) * L.Cin + ci) * 9 + bu % 9] = v;
}

// Stage 1: sum the splits.  A block covers 32 consecutive elements x 8 interleaved split groups;
// each thread adds its splits in ascending order, the groups are combined in a fixed tree, so
// the result does not depend on scheduling.  out[e] = sum_split partial[split][e].
template <bool RELAYOUT>
__global__ __launch_bounds__(256) void k_p4_sum_splits(const float* __restrict__ partial, float* __restrict__ out,
                                                       int n_elem, int splits, DwLayout L) {
  __shared__ float red[8][32];
  const int e = blockIdx.x * 32 + (threadIdx.x % 32);
  const int grp = threadIdx.x / 32;
  float s = 0.f;
  if (e < n_elem)
    for (int sp = grp; sp < splits; sp += 8) s += partial[(size_t)sp * n_elem + e];
  red[grp][threadIdx.x % 32] = s;
  __syncthreads();
  if (grp == 0 && e < n_elem) {
    const int l = threadIdx.x;
    put_sum<RELAYOUT>(out, e, ((red[0][l] + red[1][l]) + (red[2][l] + red[3][l])) + ((red[4][l] + red[5][l]) + (red[6][l] + red[7][l])), L);
  }
}

// The same sum for large images (many elements, few splits): one thread per four elements adds the splits in
// ascending order, every access a full 16-byte lane access.
template <bool RELAYOUT>
__global__ __launch_bounds__(256) void k_p4_sum_splits_wide(const float* __restrict__ partial, float* __restrict__ out,
                                                            int n4, int splits, DwLayout L) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= n4) return;
  const f4* src = reinterpret_cast<const f4*>(partial);
  f4 s = src[e];
  for (int sp = 1; sp < splits; ++sp) s += src[(size_t)sp * n4 + e];
  if (!RELAYOUT) {
    reinterpret_cast<f4*>(out)[e] = s;
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) put_sum<true>(out, 4 * e + i, s[i], L);
  }
}

// Stage 2: the transposed first-quadrant expansion (Eq. 16 / adjoint of Eq. 17):
// dw[b][co][ci][ub] = sum_z coef_z * dF[q_z][t_z][co][ci].
__global__ __launch_bounds__(256) void k_p4_reduce_w(const float* __restrict__ dF, float* __restrict__ dw,
                                                     const int32_t* __restrict__ fqt_ptr,
                                                     const int32_t* __restrict__ fqt_col,
                                                     const float* __restrict__ fqt_coef, int B, int Cout, int Cin,
                                                     int CoutPad, int CinPad, int base) {
  // one thread per (bank, filter, channel): its nine taps are nine consecutive floats of dw
  const int total = B * Cout * Cin;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int ci = e % Cin;
  const int co = (e / Cin) % Cout;
  const int b = e / (Cin * Cout);
  const size_t plane = (size_t)CoutPad * CinPad;
  const float* src = dF + (size_t)co * CinPad + ci;
  float* dst = dw + (size_t)e * 9;
#pragma unroll
  for (int ub = 0; ub < 9; ++ub) {
    float acc = 0.f;
    if (base) {       // dF already is the base banks' gradient: only the layout changes
      acc = src[(size_t)(b * 9 + ub) * plane];
    } else {
      for (int z = fqt_ptr[b * 9 + ub]; z < fqt_ptr[b * 9 + ub + 1]; ++z) acc += fqt_coef[z] * src[(size_t)fqt_col[z] * plane];
    }
    dst[ub] = acc;
  }
}

}  // namespace

bool p4_bwd_weight_supported(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  if (d.k != 3 || d.stride != 1 || d.pad != 1) return false;   // bf16 plans run these kernels on widened copies
  if (d.W & 3) return false;
  return p4_fwd_pool_mode(p) != kOutUnpooled;
}

P4BwdWGeom p4_bwd_weight_geom(const rotconv_plan* p, bool lut, bool share) {
  const rotconv_desc& d = p->d;
  P4BwdWGeom g{};
  g.N = d.N; g.Cin = d.Cin; g.H = d.H; g.W = d.W; g.Cout = d.Cout; g.Q = lut ? p->B : p->host.Q; g.ng = p->ng;
  g.lut = lut ? 1 : 0; g.R = d.R;
  g.ncb = d.Cin <= 16 ? 1 : 4;
  const int NCB = g.ncb;
  g.CinPad = (d.Cin + 16 * NCB - 1) / (16 * NCB) * (16 * NCB);
  g.CoutPad = (d.Cout + 15) / 16 * 16;
  g.ncig = g.CinPad / (16 * NCB);
  // channel groups whose waves build a filter block's D together (the bf16 table kernel; elsewhere one).  Measured
  // on the 512 x 512 stack: four groups of 64 channels 0.145 ms against 0.21 ms unshared; groups of 32 channels with
  // eight waves (two per SIMD) 0.19 ms: the sharing factor outweighs the occupancy
  g.ncg = share && lut ? (g.ncig >= 3 ? 4 : g.ncig == 2 ? 2 : 1) : 1;
  g.ncigw = (g.ncig + g.ncg - 1) / g.ncg;
  const int nfb_wg = NWAVE / g.ncg;                          // (bank, 16-filter block) pairs per workgroup
  g.ncog = (g.Q * (g.CoutPad / 16) + nfb_wg - 1) / nfb_wg;   // workgroups per channel-group set and split
  // work units: (image, row range, 32-pixel strip); a range never crosses an image
  const int combos = g.ncigw * g.ncog;
  g.nstrip = (d.W + 31) / 32;
  // units wanted to fill the chip: one workgroup per CU; two where the instance leaves room for two waves per SIMD
  // (one channel block per wave: the first layer)
  const int fill = (NCB == 1 && !(lut && p->d.dtype != ROTCONV_BF16)) ? 512 : 256;
  const int want = (fill + combos - 1) / combos;
  int per_image = std::max(1, std::min(d.H, (want + d.N * g.nstrip - 1) / (d.N * g.nstrip)));
  g.rows_per = (d.H + per_image - 1) / per_image;
  g.nrange = (d.H + g.rows_per - 1) / g.rows_per;
  g.units = d.N * g.nrange * g.nstrip;
  // one partial-sum image per split; keep them below 256 MiB (a workgroup then takes several units)
  const double per = 4.0 * g.Q * 9.0 * g.CoutPad * g.CinPad;
  g.splits = std::max(1, std::min(std::min(g.units, want), (int)(268435456.0 / per)));
  return g;
}

// The bf16 kernel loads a lane's 8 pixels with one 16-byte access: rows must start 16-byte aligned.
bool p4_bwd_weight_bf16_supported(const rotconv_plan* p) { return p4_bwd_weight_supported(p) && (p->d.W & 7) == 0; }

size_t p4_bwd_weight_ws_floats(const rotconv_plan* p) {
  size_t need = 0;
  for (int lut = 0; lut < 3; ++lut) {     // the per-bank kernels (also the bf16 one), the table variant, its shared-D form
    if (lut && !p4_bwd_lut(p) && !p->bwd_lut16[2]) break;
    const P4BwdWGeom g = p4_bwd_weight_geom(p, lut != 0, lut == 2);
    need = std::max(need, (size_t)(g.splits + 1) * g.Q * 9 * g.CoutPad * g.CinPad);  // partial sums + their total
  }
  return need;
}

// partial sums of the splits -> dF (fixed order) -> dw through the transposed expansion; one launch where that
// expansion is the identity
static bool dw_is_relayout(const rotconv_plan* p, const P4BwdWGeom& g) {
  if (g.lut) return true;
  if (g.Q != 1 || p->B != 1) return false;
  for (int u = 0; u < 9; ++u)
    for (int z = 0; z < kMaxNnz; ++z) {
      const int src = p->host.fq_src[u * kMaxNnz + z];
      if (z == 0 ? (src != u || p->host.fq_coef[u * kMaxNnz] != 1.0f) : src >= 0) return false;
    }
  return true;
}
static void finish_dw(const rotconv_plan* p, const P4BwdWGeom& g, float* partial, float* dw, hipStream_t st) {
  const int n_elem = g.Q * 9 * g.CoutPad * g.CinPad;      // a multiple of 16
  const DwLayout L{g.Cout, g.Cin, g.CoutPad, g.CinPad};
  const bool relayout = g.splits > 1 && dw_is_relayout(p, g);
  float* dF = partial;                                     // a single split is the sum
  if (g.splits > 1) {
    dF = relayout ? dw : partial + (size_t)g.splits * n_elem;
    if (n_elem >= (1 << 18)) {
      if (relayout) hipLaunchKernelGGL(k_p4_sum_splits_wide<true>, dim3((n_elem / 4 + 255) / 256), dim3(256), 0, st, partial, dF, n_elem / 4, g.splits, L);
      else hipLaunchKernelGGL(k_p4_sum_splits_wide<false>, dim3((n_elem / 4 + 255) / 256), dim3(256), 0, st, partial, dF, n_elem / 4, g.splits, L);
    } else {
      if (relayout) hipLaunchKernelGGL(k_p4_sum_splits<true>, dim3((n_elem + 31) / 32), dim3(256), 0, st, partial, dF, n_elem, g.splits, L);
      else hipLaunchKernelGGL(k_p4_sum_splits<false>, dim3((n_elem + 31) / 32), dim3(256), 0, st, partial, dF, n_elem, g.splits, L);
    }
    if (relayout) return;
  }
  const int total = p->B * g.Cout * g.Cin;
  hipLaunchKernelGGL(k_p4_reduce_w, dim3((total + 255) / 256), dim3(256), 0, st, dF, dw, p->dev.fqt_ptr,
                     p->dev.fqt_col, p->dev.fqt_coef, p->B, g.Cout, g.Cin, g.CoutPad, g.CinPad, g.lut);
}

void launch_p4_bwd_weight(const rotconv_plan* p, const float* x, const float* gpool, const uint8_t* idx,
                          float* partial, float* dw, hipStream_t st) {
  const P4BwdWGeom g = p4_bwd_weight_geom(p, p4_bwd_lut(p), true);
  const int grid = g.splits * g.ncigw * g.ncog;
  if (g.ncg > 1) {          // table variant, the channel groups of a filter block build its D together
    auto gos = [&](auto kern) {
      const size_t lds = ((size_t)2 * 9 * 33 * 12 + (size_t)2 * (NWAVE / g.ncg) * 9 * 16 * 36) * sizeof(float);
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), lds, st, x, gpool, idx, p->dev.lut_bwd, partial, g);
    };
    if (g.ncg == 4) gos(k_p4_bwd_weight_lut_shared<4>);
    else gos(k_p4_bwd_weight_lut_shared<2>);
    finish_dw(p, g, partial, dw, st);
    return;
  }
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), 0, st, x, gpool, idx, p->dev.rot_of, p->dev.lut_bwd, partial, g);
  };
  if (g.ncb == 1) { if (g.lut) go(k_p4_bwd_weight<1, true>); else go(k_p4_bwd_weight<1, false>); }
  else { if (g.lut) go(k_p4_bwd_weight<4, true>); else go(k_p4_bwd_weight<4, false>); }
  finish_dw(p, g, partial, dw, st);
}

void launch_p4_bwd_weight_bf16(const rotconv_plan* p, const uint16_t* x, const uint16_t* gpool, const uint8_t* idx,
                               float* partial, float* dw, hipStream_t st) {
  if (p->bwd_lut16[2]) {      // routed-gradient table: one contraction with the base bank
    const P4BwdWGeom g = p4_bwd_weight_geom(p, true, true);
    const int grid = g.splits * g.ncigw * g.ncog;
    if (g.ncg > 1) {          // the channel groups of a filter block build its D together
      auto go = [&](auto kern, int nw) {
        const size_t lds = (size_t)2 * 9 * 33 * 12 * 4 + (size_t)2 * (nw / g.ncg) * 9 * 16 * 16 * 4;
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * nw), lds, st, x, gpool, idx, p->dev.lut_bwd, partial, g);
      };
      if (g.ncg == 4) go(k_p4_bwd_weight_bf16_lut_shared<4, 4, 4>, 4);
      else go(k_p4_bwd_weight_bf16_lut_shared<4, 2, 4>, 4);
      finish_dw(p, g, partial, dw, st);
      return;
    }
    if (g.ncb == 1) hipLaunchKernelGGL(k_p4_bwd_weight_bf16_lut<1>, dim3(grid), dim3(NT), 0, st, x, gpool, idx, p->dev.lut_bwd, partial, g);
    else hipLaunchKernelGGL(k_p4_bwd_weight_bf16_lut<4>, dim3(grid), dim3(NT), 0, st, x, gpool, idx, p->dev.lut_bwd, partial, g);
    finish_dw(p, g, partial, dw, st);
    return;
  }
  const P4BwdWGeom g = p4_bwd_weight_geom(p);
  const int grid = g.splits * g.ncig * g.ncog;
  if (g.ncb == 1) hipLaunchKernelGGL(k_p4_bwd_weight_bf16<1>, dim3(grid), dim3(NT), 0, st, x, gpool, idx, p->dev.rot_of, partial, g);
  else hipLaunchKernelGGL(k_p4_bwd_weight_bf16<4>, dim3(grid), dim3(NT), 0, st, x, gpool, idx, p->dev.rot_of, partial, g);
  finish_dw(p, g, partial, dw, st);
}

}  // namespace rotconv
