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
// channels, K = 4 pixels; D is built on the fly by selects and adds in the A-operand
// layout (a lane owns 4 consecutive pixels of one filter and reads the 3x6
// neighbourhood of (G, idx) around them), X goes straight from global memory into
// the B operand.  A wave keeps the 9 x 4 accumulator tiles of its 16 filters x 64
// channels (144 registers) over its whole pixel range; ranges ("splits") are
// summed afterwards in a fixed order by the reduction kernel, which also applies
// the transposed first-quadrant expansion, so the result is deterministic.
#include <hip/hip_runtime.h>

#include "rotconv_kernels.h"
#include "rotconv_p4.h"

namespace rotconv {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int NCB = 4;         // 16-channel blocks per wave (64 input channels)
constexpr int NWAVE = 4;       // waves per workgroup = 16-filter blocks per workgroup
constexpr int NT = 64 * NWAVE;

__device__ __host__ constexpr int tap_i(int s, int u) {
  return s == 0 ? u / 3 : s == 1 ? 2 - u % 3 : s == 2 ? 2 - u / 3 : u % 3;
}
__device__ __host__ constexpr int tap_j(int s, int u) {
  return s == 0 ? u % 3 : s == 1 ? u / 3 : s == 2 ? 2 - u % 3 : 2 - u / 3;
}

struct RawW {            // (G, idx) of one filter on a 3 x 6 pixel neighbourhood
  float g[3][6];
  uint32_t ic[3];        // idx bytes of the 4 centre pixels
  uint32_t ie[3];        // byte 0: left neighbour, byte 1: right neighbour
};

__global__ __launch_bounds__(NT) void k_p4_bwd_weight(const float* __restrict__ x, const float* __restrict__ gpool,
                                                      const uint8_t* __restrict__ idx,
                                                      const int32_t* __restrict__ rot_of,
                                                      float* __restrict__ partial, P4BwdWGeom g) {
  int v = blockIdx.x;
  const int split = v % g.splits; v /= g.splits;
  const int cig = v % g.ncig; v /= g.ncig;
  const int cog = v % g.ncog;
  const int q = v / g.ncog;

  const int tid = threadIdx.x;
  const int wave = tid / 64, lane = tid % 64;
  const int lg = lane / 16, lc = lane % 16;
  const int HW = g.H * g.W;
  const int co = (cog * NWAVE + wave) * 16 + lc;     // this lane's filter (A role)
  const int ci0 = cig * 16 * NCB + lc;               // this lane's channel in block 0 (B role)

  int rot[4];
  int r0 = -1;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    rot[s] = rot_of[q * 4 + s];
    if (r0 < 0 && rot[s] >= 0) r0 = rot[s];
  }
  const bool cok = co < g.Cout && r0 >= 0;
  const size_t gplane0 = ((size_t)(cok ? co : 0) * g.ng + (r0 < 0 ? 0 : r0 % g.ng)) * HW;
  const size_t gimg = (size_t)g.Cout * g.ng * HW;

  // rows of the flattened (n, h) space handled by this split
  const int rows_total = g.N * g.H;
  const int rows_per = (rows_total + g.splits - 1) / g.splits;
  const int row_begin = split * rows_per;
  const int row_end = min(rows_total, row_begin + rows_per);
  const int w16 = (g.W + 15) / 16;
  const int nrows = max(0, row_end - row_begin);
  const int niter = nrows * w16;

  // Branch-free loads (out-of-range positions read a safe address and are masked; an idx byte of
  // 0xff matches no orientation), so that a pipeline stage is one basic block.
  auto load_b = [&](int it, f4 (&b)[NCB]) {
    it = min(it, niter - 1);
    const int row = row_begin + it % nrows;   // rows run fastest: (G, idx) rows are re-read from L1
    const int n = row / g.H, h = row % g.H;
    const int px = (it / nrows) * 16 + 4 * lg;
    const bool pok = px < g.W;                // W % 4 == 0: the four pixels are in or out together
    const size_t off = (size_t)n * g.Cin * HW + (size_t)h * g.W + (pok ? px : 0);
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      const int ci = ci0 + cb * 16;
      const bool ok = pok && ci < g.Cin;
      const f4 val = *reinterpret_cast<const f4*>(x + off + (size_t)(ci < g.Cin ? ci : 0) * HW);
      b[cb] = ok ? val : f4{0.f, 0.f, 0.f, 0.f};
    }
  };
  auto load_raw = [&](int it, RawW& r) {
    it = min(it, niter - 1);
    const int row = row_begin + it % nrows;
    const int n = row / g.H, h = row % g.H;
    const int px = (it / nrows) * 16 + 4 * lg;
    const bool pok = px < g.W;
    const int pc = pok ? px : 0, pl = max(px - 1, 0), pr = min(px + 4, g.W - 1);
    const bool lok = px >= 1 && px - 1 < g.W, rok2 = px + 4 < g.W;
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      const int rr = h - 1 + dr;
      const bool rok = cok && rr >= 0 && rr < g.H;
      const size_t rowbase = (size_t)n * gimg + gplane0 + (size_t)(rok ? rr : 0) * g.W;
      const f4 gc = *reinterpret_cast<const f4*>(gpool + rowbase + pc);
      const uint32_t ic = *reinterpret_cast<const uint32_t*>(idx + rowbase + pc);
      const float gl = gpool[rowbase + pl], gr = gpool[rowbase + pr];
      const uint32_t il = idx[rowbase + pl], ir = idx[rowbase + pr];
      r.g[dr][1] = gc[0]; r.g[dr][2] = gc[1]; r.g[dr][3] = gc[2]; r.g[dr][4] = gc[3];
      r.g[dr][0] = gl;
      r.g[dr][5] = gr;
      r.ic[dr] = (rok && pok) ? ic : 0xffffffffu;
      r.ie[dr] = ((rok && lok) ? il : 0xffu) | (((rok && rok2) ? ir : 0xffu) << 8);
    }
  };

  // One quarter turn's share of D for the lane's four pixels: Delta_s on the 3x6 neighbourhood,
  // added where R_s puts each base tap (Eq. 12 with the tap positions of Eq. 8).
  auto build_slice = [&](const RawW& r, int s, float (&a)[9][4]) {
    const uint32_t rs = (uint32_t)rot[s];     // -1 (absent) matches no byte
    float d[3][6];
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
      d[dr][0] = ((r.ie[dr] & 0xffu) == rs) ? r.g[dr][0] : 0.f;
      d[dr][5] = (((r.ie[dr] >> 8) & 0xffu) == rs) ? r.g[dr][5] : 0.f;
#pragma unroll
      for (int p = 0; p < 4; ++p) d[dr][1 + p] = (((r.ic[dr] >> (8 * p)) & 0xffu) == rs) ? r.g[dr][1 + p] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 9; ++u)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const float term = d[2 - tap_i(s, u)][t + 2 - tap_j(s, u)];
        a[u][t] = s == 0 ? term : a[u][t] + term;
      }
  };

  f4 acc[9][NCB];
#pragma unroll
  for (int u = 0; u < 9; ++u)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[u][cb] = f4{0.f, 0.f, 0.f, 0.f};

  if (niter > 0) {
    // Three-stage software pipeline, unrolled twice so that no buffer is copied: loads of (G, idx)
    // for step it+2 and of X for step it+1; D build for step it+1, one quarter turn after each of
    // the four K-steps of step it, so that the VALU work sits between the MFMAs.
    RawW rawA, rawB;
    f4 bA[NCB], bB[NCB];
    float aA[9][4], aB[9][4];
    auto stage = [&](int it, const RawW& raw_use, RawW& raw_ld, const float (&a_cur)[9][4], float (&a_nxt)[9][4],
                     const f4 (&b_cur)[NCB], f4 (&b_nxt)[NCB]) {
      load_raw(it + 2, raw_ld);
      load_b(it + 1, b_nxt);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
#pragma unroll
        for (int u = 0; u < 9; ++u)
#pragma unroll
          for (int cb = 0; cb < NCB; ++cb)
            acc[u][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[u][t], b_cur[cb][t], acc[u][cb], 0, 0, 0);
        build_slice(raw_use, t, a_nxt);
      }
    };
    load_raw(0, rawB);
    load_b(0, bA);
#pragma unroll
    for (int s = 0; s < 4; ++s) build_slice(rawB, s, aA);
    load_raw(1, rawA);
    for (int it = 0; it < niter; it += 2) {
      stage(it, rawA, rawB, aA, aB, bA, bB);
      if (it + 1 < niter) stage(it + 1, rawB, rawA, aB, aA, bB, bA);
    }
  }

  // partial[split][q][u][CoutPad][CinPad]; lane holds rows (filters) 4*lg+i, column (channel) lc
  const int cobase = (cog * NWAVE + wave) * 16;
  if (cobase < g.CoutPad) {
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

// Stage 1: sum the splits.  A block covers 32 consecutive elements x 8 interleaved split groups;
// each thread adds its splits in ascending order, the groups are combined in a fixed tree, so
// the result does not depend on scheduling.  out[e] = sum_split partial[split][e].
__global__ __launch_bounds__(256) void k_p4_sum_splits(const float* __restrict__ partial, float* __restrict__ out,
                                                       int n_elem, int splits) {
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
    out[e] = ((red[0][l] + red[1][l]) + (red[2][l] + red[3][l])) + ((red[4][l] + red[5][l]) + (red[6][l] + red[7][l]));
  }
}

// Stage 2: the transposed first-quadrant expansion (Eq. 16 / adjoint of Eq. 17):
// dw[b][co][ci][ub] = sum_z coef_z * dF[q_z][t_z][co][ci].
__global__ __launch_bounds__(256) void k_p4_reduce_w(const float* __restrict__ dF, float* __restrict__ dw,
                                                     const int32_t* __restrict__ fqt_ptr,
                                                     const int32_t* __restrict__ fqt_col,
                                                     const float* __restrict__ fqt_coef, int B, int Cout, int Cin,
                                                     int CoutPad, int CinPad) {
  const int total = B * 9 * Cout * Cin;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int ci = e % Cin;
  const int co = (e / Cin) % Cout;
  const int ub = (e / (Cin * Cout)) % 9;
  const int b = e / (Cin * Cout * 9);
  const size_t plane = (size_t)CoutPad * CinPad;
  float acc = 0.f;
  for (int z = fqt_ptr[b * 9 + ub]; z < fqt_ptr[b * 9 + ub + 1]; ++z)
    acc += fqt_coef[z] * dF[(size_t)fqt_col[z] * plane + (size_t)co * CinPad + ci];
  dw[(((size_t)b * Cout + co) * Cin + ci) * 9 + ub] = acc;
}

}  // namespace

bool p4_bwd_weight_supported(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  if (d.k != 3 || d.stride != 1 || d.pad != 1 || d.dtype != ROTCONV_F32) return false;
  if (d.W & 3) return false;
  return p4_fwd_pool_mode(p) != kOutUnpooled;
}

P4BwdWGeom p4_bwd_weight_geom(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  P4BwdWGeom g{};
  g.N = d.N; g.Cin = d.Cin; g.H = d.H; g.W = d.W; g.Cout = d.Cout; g.Q = p->host.Q; g.ng = p->ng;
  g.CinPad = (d.Cin + 16 * NCB - 1) / (16 * NCB) * (16 * NCB);
  g.CoutPad = (d.Cout + 16 * NWAVE - 1) / (16 * NWAVE) * (16 * NWAVE);
  g.ncig = g.CinPad / (16 * NCB);
  g.ncog = g.CoutPad / (16 * NWAVE);
  const int combos = g.Q * g.ncig * g.ncog;
  const int rows = d.N * d.H;
  int splits = (256 + combos - 1) / combos;
  splits = std::min(splits, rows);
  // keep the partial sums below 256 MiB
  const double per = 4.0 * g.Q * 9.0 * g.CoutPad * g.CinPad;
  splits = std::max(1, std::min(splits, (int)(268435456.0 / per)));
  // equal row counts per split where possible
  const int rows_per = (rows + splits - 1) / splits;
  g.splits = (rows + rows_per - 1) / rows_per;
  return g;
}

size_t p4_bwd_weight_ws_floats(const rotconv_plan* p) {
  const P4BwdWGeom g = p4_bwd_weight_geom(p);
  return (size_t)(g.splits + 1) * g.Q * 9 * g.CoutPad * g.CinPad;  // partial sums + their total
}

void launch_p4_bwd_weight(const rotconv_plan* p, const float* x, const float* gpool, const uint8_t* idx,
                          float* partial, float* dw, hipStream_t st) {
  const P4BwdWGeom g = p4_bwd_weight_geom(p);
  const int grid = g.splits * g.ncig * g.ncog * g.Q;
  hipLaunchKernelGGL(k_p4_bwd_weight, dim3(grid), dim3(NT), 0, st, x, gpool, idx, p->dev.rot_of, partial, g);
  const int n_elem = g.Q * 9 * g.CoutPad * g.CinPad;
  float* dF = partial + (size_t)g.splits * n_elem;
  hipLaunchKernelGGL(k_p4_sum_splits, dim3((n_elem + 31) / 32), dim3(256), 0, st, partial, dF, n_elem, g.splits);
  const int total = p->B * 9 * g.Cout * g.Cin;
  hipLaunchKernelGGL(k_p4_reduce_w, dim3((total + 255) / 256), dim3(256), 0, st, dF, dw, p->dev.fqt_ptr,
                     p->dev.fqt_col, p->dev.fqt_coef, p->B, g.Cout, g.Cin, g.CoutPad, g.CinPad);
}

}  // namespace rotconv
