// Host logic of the rotation-convolution library: descriptor validation and the
// orientation tables: per (rotation, tap) the output position of every product and the
// expansion coefficients, computed once per plan (paper Sec. III-B, Eq. 8; Sec. III-D).
// No GPU calls in this file.
#include <cmath>
#include <cstring>
#include <new>

#include "rotconv_internal.h"

namespace rotconv {
namespace {

constexpr double kPi = 3.141592653589793238462643383279502884;

struct Nz {
  int src;      // b*kk + u
  double coef;
};

// Where base tap u = (m,n) sits after s counter-clockwise quarter turns of a k x k filter.
// One turn sends (m,n) to (k-1-n, m)  [rot90(A)[i][j] = A[j][k-1-i]].
int turned_tap(int k, int s, int u) {
  int m = u / k, n = u % k;
  for (int q = 0; q < s; ++q) {
    const int mm = k - 1 - n;
    n = m;
    m = mm;
  }
  return m * k + n;
}

// Non-zeros of row (dst tap t) of the first-quadrant map base -> F_phi.
// mirrored: the bank is built from the left-right mirrored base filter (P4M mode: a tap permutation).
int first_quadrant_row(int mode, int k, double phi_deg, bool mirrored, int t, Nz out[kMaxNnz]) {
  const int kk = k * k;
  if (mode == ROTCONV_P4M) {
    out[0] = {mirrored ? (t / k) * k + (k - 1 - t % k) : t, 1.0};
    return 1;
  }
  if (mode == ROTCONV_EXACT90 || (mode == ROTCONV_BILINEAR && phi_deg == 0.0)) {
    out[0] = {t, 1.0};
    return 1;
  }
  const double phi = phi_deg * kPi / 180.0;
  if (mode == ROTCONV_STEERABLE) {  // Eq. 17
    out[0] = {t, std::sin(phi)};
    out[1] = {kk + t, std::cos(phi)};
    return 2;
  }
  // BILINEAR: the value of F_phi at grid offset (dr,dc) from the centre is the base filter
  // sampled at that offset turned back by phi; rows grow downwards, so in (row,col) terms
  //   dr_s = cos(phi) dr + sin(phi) dc,   dc_s = -sin(phi) dr + cos(phi) dc.
  const double c = 0.5 * (k - 1);
  const double dr = t / k - c, dc = t % k - c;
  const double rs = c + std::cos(phi) * dr + std::sin(phi) * dc;
  const double cs = c - std::sin(phi) * dr + std::cos(phi) * dc;
  const double r0 = std::floor(rs), c0 = std::floor(cs);
  const double fr = rs - r0, fc = cs - c0;
  int n = 0;
  for (int a = 0; a < 2; ++a)
    for (int b = 0; b < 2; ++b) {
      const int rr = static_cast<int>(r0) + a, cc = static_cast<int>(c0) + b;
      if (rr < 0 || rr >= k || cc < 0 || cc >= k) continue;
      const double wv = (a ? fr : 1.0 - fr) * (b ? fc : 1.0 - fc);
      if (wv == 0.0) continue;
      out[n++] = {rr * k + cc, wv};
    }
  return n;
}

void build_csr_transpose(int rows_out, int n_rows_in, const std::vector<int32_t>& src, const std::vector<float>& coef,
                         std::vector<int32_t>* ptr, std::vector<int32_t>* col, std::vector<float>* val) {
  ptr->assign(rows_out + 1, 0);
  for (int row = 0; row < n_rows_in; ++row)
    for (int e = 0; e < kMaxNnz; ++e) {
      const int s = src[row * kMaxNnz + e];
      if (s >= 0) (*ptr)[s + 1]++;
    }
  for (int i = 0; i < rows_out; ++i) (*ptr)[i + 1] += (*ptr)[i];
  col->assign((*ptr)[rows_out], 0);
  val->assign((*ptr)[rows_out], 0.f);
  std::vector<int32_t> fill(ptr->begin(), ptr->end() - 1);
  for (int row = 0; row < n_rows_in; ++row)  // ascending input row => deterministic order
    for (int e = 0; e < kMaxNnz; ++e) {
      const int s = src[row * kMaxNnz + e];
      if (s < 0) continue;
      (*col)[fill[s]] = row;
      (*val)[fill[s]] = coef[row * kMaxNnz + e];
      fill[s]++;
    }
}

bool fits_i32(double v) { return v < 2147483647.0; }

}  // namespace

int validate_and_build(const rotconv_desc* desc, rotconv_plan** out) {
  if (!desc || !out) return ROTCONV_ERR_NULL;
  const rotconv_desc& d = *desc;
  if (d.N < 1 || d.Cin < 1 || d.H < 1 || d.W < 1 || d.Cout < 1 || d.k < 1) return ROTCONV_ERR_SHAPE;
  if (d.R < 1 || d.R > 255) return ROTCONV_ERR_SHAPE;
  if (d.stride < 1 || d.pad < 0) return ROTCONV_ERR_SHAPE;
  if (d.pool_group < 0) return ROTCONV_ERR_SHAPE;
  const int G = d.pool_group == 0 ? d.R : d.pool_group;
  if (G > d.R || d.R % G != 0) return ROTCONV_ERR_SHAPE;
  if (d.H + 2 * d.pad < d.k || d.W + 2 * d.pad < d.k) return ROTCONV_ERR_SHAPE;
  if (d.mode != ROTCONV_EXACT90 && d.mode != ROTCONV_STEERABLE && d.mode != ROTCONV_BILINEAR && d.mode != ROTCONV_P4M)
    return ROTCONV_ERR_UNSUPPORTED;
  const bool p4m = d.mode == ROTCONV_P4M;
  if (p4m && (d.angles_deg || (d.R != 2 && d.R != 4 && d.R != 8))) return ROTCONV_ERR_ANGLES;
  if (d.dtype != ROTCONV_F32 && d.dtype != ROTCONV_BF16) return ROTCONV_ERR_UNSUPPORTED;
  if (d.pool_op != ROTCONV_POOL_MAX && d.pool_op != ROTCONV_POOL_AVG) return ROTCONV_ERR_UNSUPPORTED;
  if (d.activation != ROTCONV_ACT_NONE && d.activation != ROTCONV_ACT_RELU) return ROTCONV_ERR_UNSUPPORTED;
  if (d.activation == ROTCONV_ACT_RELU && d.pool_op != ROTCONV_POOL_MAX) return ROTCONV_ERR_UNSUPPORTED;
  if (d.k > 15) return ROTCONV_ERR_UNSUPPORTED;
  // the general kernels put a channel extent into the grid's y dimension and the batch into z (65535 each)
  if ((long long)d.Cout * d.R > 65535 || d.Cin > 65535 || d.N > 65535) return ROTCONV_ERR_UNSUPPORTED;
  const int Ho = (d.H + 2 * d.pad - d.k) / d.stride + 1, Wo = (d.W + 2 * d.pad - d.k) / d.stride + 1;
  const int kk = d.k * d.k, B = d.mode == ROTCONV_STEERABLE ? 2 : 1;
  // Kernels index every tensor with 32-bit element offsets.
  if (!fits_i32(double(d.N) * d.Cin * d.H * d.W) || !fits_i32(double(d.N) * d.Cout * d.R * Ho * Wo) ||
      !fits_i32(double(d.R) * d.Cout * d.Cin * kk))
    return ROTCONV_ERR_UNSUPPORTED;

  // P4M: the second half of the orientations repeats the angles of the first on the mirrored filter
  const int nrot = p4m ? d.R / 2 : d.R;
  std::vector<double> ang(d.R);
  for (int r = 0; r < d.R; ++r) ang[r] = d.angles_deg ? d.angles_deg[r] : (r % nrot) * (360.0 / nrot);
  for (int r = 0; r < d.R; ++r) {
    if (!(ang[r] >= 0.0 && ang[r] < 360.0)) return ROTCONV_ERR_ANGLES;
    if (r % nrot && !(ang[r] > ang[r - 1])) return ROTCONV_ERR_ANGLES;
    if ((d.mode == ROTCONV_EXACT90 || p4m) && std::fmod(ang[r], 90.0) != 0.0) return ROTCONV_ERR_ANGLES;
  }

  rotconv_plan* p = new (std::nothrow) rotconv_plan();
  if (!p) return ROTCONV_ERR_LAUNCH;
  p->d = d;
  p->angles = ang;
  p->d.angles_deg = p->angles.data();
  p->d.pool_group = G;
  p->B = B;
  p->G = G;
  p->ng = d.R / G;
  p->Ho = Ho;
  p->Wo = Wo;
  p->kk = kk;

  HostTables& t = p->host;
  t.bank_of_r.resize(d.R);
  t.quarter_of_r.resize(d.R);
  for (int r = 0; r < d.R; ++r) {
    const int s = static_cast<int>(std::floor(ang[r] / 90.0));
    const double phi = ang[r] - 90.0 * s;
    const int mir = p4m && r >= nrot ? 1 : 0;
    int q = -1;
    for (size_t i = 0; i < t.phi_deg.size(); ++i)
      if (t.phi_deg[i] == phi && t.mirrored[i] == mir) q = static_cast<int>(i);
    if (q < 0) {
      q = static_cast<int>(t.phi_deg.size());
      t.phi_deg.push_back(phi);
      t.mirrored.push_back(mir);
    }
    t.bank_of_r[r] = q;
    t.quarter_of_r[r] = s & 3;
  }
  t.Q = static_cast<int>(t.phi_deg.size());
  p->rot_of.assign(t.Q * 4, -1);
  for (int r = 0; r < d.R; ++r) p->rot_of[t.bank_of_r[r] * 4 + t.quarter_of_r[r]] = r;

  t.turn_tap.resize(4 * kk);
  for (int s = 0; s < 4; ++s)
    for (int u = 0; u < kk; ++u) t.turn_tap[s * kk + u] = turned_tap(d.k, s, u);

  t.fq_src.assign(t.Q * kk * kMaxNnz, -1);
  t.fq_coef.assign(t.Q * kk * kMaxNnz, 0.f);
  t.fq_coef64.assign(t.Q * kk * kMaxNnz, 0.0);
  for (int q = 0; q < t.Q; ++q)
    for (int u = 0; u < kk; ++u) {
      Nz nz[kMaxNnz];
      const int n = first_quadrant_row(d.mode, d.k, t.phi_deg[q], t.mirrored[q] != 0, u, nz);
      for (int e = 0; e < n; ++e) {
        t.fq_src[(q * kk + u) * kMaxNnz + e] = nz[e].src;
        t.fq_coef[(q * kk + u) * kMaxNnz + e] = static_cast<float>(nz[e].coef);
        t.fq_coef64[(q * kk + u) * kMaxNnz + e] = nz[e].coef;
      }
    }
  // W^(r)[R_s(u)] = F_phi[u]: the row of first-quadrant tap u becomes the row of its turned tap.
  t.exp_src.assign(d.R * kk * kMaxNnz, -1);
  t.exp_coef.assign(d.R * kk * kMaxNnz, 0.f);
  t.exp_coef64.assign(d.R * kk * kMaxNnz, 0.0);
  for (int r = 0; r < d.R; ++r)
    for (int u = 0; u < kk; ++u) {
      const int dst = t.turn_tap[t.quarter_of_r[r] * kk + u];
      for (int e = 0; e < kMaxNnz; ++e) {
        t.exp_src[(r * kk + dst) * kMaxNnz + e] = t.fq_src[(t.bank_of_r[r] * kk + u) * kMaxNnz + e];
        t.exp_coef[(r * kk + dst) * kMaxNnz + e] = t.fq_coef[(t.bank_of_r[r] * kk + u) * kMaxNnz + e];
        t.exp_coef64[(r * kk + dst) * kMaxNnz + e] = t.fq_coef64[(t.bank_of_r[r] * kk + u) * kMaxNnz + e];
      }
    }
  if (kk == 9) {
    t.fq_dense64.assign((size_t)t.Q * 9 * B * 9, 0.0);
    for (int q = 0; q < t.Q; ++q)
      for (int u = 0; u < 9; ++u)
        for (int e = 0; e < kMaxNnz; ++e) {
          const int src = t.fq_src[(q * 9 + u) * kMaxNnz + e];
          if (src >= 0) t.fq_dense64[((size_t)q * 9 + u) * (B * 9) + src] += t.fq_coef64[(q * 9 + u) * kMaxNnz + e];
        }
  }
  // 3x3: the routed-gradient table of the input / weight gradients.  With Delta_r = G [idx == r]
  // (Eq. 12) the gradient that reaches base tap u' from the neighbour at offset (dy, dx) of a pixel is
  // G * lut[(dy+1)*3 + (dx+1)][idx][u'], lut[.][r][u'] = coefficient of base tap u' in tap (1-dy, 1-dx) of the
  // rotated bank r (Eq. 13-16 with the expansion of Eq. 5 / Sec. III-D folded in); row R (no orientation) is zero.
  // One such table per base bank (the steerable pair has two: [B][9][R + 1][12]).
  if (kk == 9) {
    t.lut_bwd.assign((size_t)B * 9 * (d.R + 1) * 12, 0.f);
    for (int r = 0; r < d.R; ++r)
      for (int tp = 0; tp < 9; ++tp) {
        const int rel = (2 - tp / 3) * 3 + (2 - tp % 3);
        for (int e = 0; e < kMaxNnz; ++e) {
          const int src = t.exp_src[(r * kk + tp) * kMaxNnz + e];      // base bank * 9 + base tap
          if (src >= 0)
            t.lut_bwd[(((size_t)(src / 9) * 9 + rel) * (d.R + 1) + r) * 12 + src % 9] += t.exp_coef[(r * kk + tp) * kMaxNnz + e];
        }
      }
  }
  build_csr_transpose(B * kk, d.R * kk, t.exp_src, t.exp_coef, &t.tr_ptr, &t.tr_col, &t.tr_coef);
  build_csr_transpose(B * kk, t.Q * kk, t.fq_src, t.fq_coef, &t.fqt_ptr, &t.fqt_col, &t.fqt_coef);

  *out = p;
  return ROTCONV_OK;
}

}  // namespace rotconv
