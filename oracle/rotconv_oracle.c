/*
 * CPU ORACLE for multi-orientation (rotation-invariant) 2-D convolution.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP library is checked against.  It shares no code, header, table or helper
 * with the HIP path and must never be called from it; only tests, the smoke
 * check and the benchmark's cpu_baseline leg may use it.
 *
 * Everything is fp64, plain nested loops, no blocking or fusion.  OpenMP is
 * used only to split the outermost independent loop across cores.
 *
 * What the method computes (paper, Sec. III): one base filter bank is expanded
 * to R orientations; every orientation is an ordinary cross-correlation
 * (Eq. 1 / Eq. 7); the paper's scatter formulation (Eq. 3, 4, 8, Alg. 1)
 * reaches exactly the same numbers, only with the multiplications shared.  So
 * the oracle is the definition itself, and a second function below follows the
 * scatter formulation step by step as a cross-check.
 *
 * Layouts (all row-major, contiguous):
 *   x      [N][Cin][H][W]
 *   w_base [B][Cout][Cin][k][k]   B = 2 (f_x, then f_y) in steerable mode, else 1
 *   w_rot  [R][Cout][Cin][k][k]   explicitly materialised rotated banks
 *   y, dy  [N][Cout][R][Ho][Wo]   (i.e. channel = co*R + r)
 *   ypool  [N][Cout][R/G][Ho][Wo] (i.e. channel = co*(R/G) + g)
 *   idx    same shape as ypool, uint8, holds the orientation index r in 0..R-1
 *
 * Readings of the paper taken here (the paper is silent or ambiguous on them):
 *   - "rotate by 90 degrees" (Eq. 5) is counter-clockwise with row 0 drawn on
 *     top: rot90(A)[i][j] = A[j][k-1-i], which is what numpy.rot90 does.
 *   - Eq. 1/7 are written for 'valid' outputs while Eq. 3/8 produce a
 *     same-size output through the floor(K/2) offset; both are the case
 *     pad = 0 resp. pad = floor(K/2) of zero padding `pad`, stride `stride`.
 *   - argmax ties (the paper writes r* "in" argmax): smallest r wins.
 *   - orientation r has angle theta_r = s_r*90 + phi_r with phi_r in [0,90);
 *     its filter is the first-quadrant filter F_phi turned by s_r exact
 *     quarter turns (Sec. III-D: only first-quadrant angles get their own
 *     filter, the other quadrants are the symmetric copies).
 *   - first-quadrant filter: steerable mode is Eq. 17; bilinear mode is a rule
 *     of this build, not the paper's (the paper avoids interpolation): inverse
 *     mapping about the tap-grid centre, zero outside the k x k support.
 *     PARITY UNPINNED by the paper for the bilinear rule itself; it is pinned
 *     against scipy.ndimage.rotate in the tests.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_EXACT90 0
#define ORC_STEERABLE 1
#define ORC_BILINEAR 2

static const double ORC_PI = 3.14159265358979323846264338327950288;

/* One exact quarter turn of a k x k array, counter-clockwise (Eq. 5 with r=1). */
static void rot90_once(const double* a, double* out, int k) {
  for (int i = 0; i < k; ++i)
    for (int j = 0; j < k; ++j) out[i * k + j] = a[j * k + (k - 1 - i)];
}

/* Inverse of the above (clockwise quarter turn): undo[j][k-1-i] = a[i][j]. */
static void rot90_undo_once(const double* a, double* out, int k) {
  for (int i = 0; i < k; ++i)
    for (int j = 0; j < k; ++j) out[j * k + (k - 1 - i)] = a[i * k + j];
}

/* Bilinear sample weights: for output tap (i,j) of the filter turned by phi
 * (counter-clockwise), the four source taps and their weights. Taps outside
 * the support get weight on a source index of -1 (caller skips them). */
static void bilinear_sources(int k, double phi_rad, int i, int j, int src[4], double wgt[4]) {
  const double c = 0.5 * (k - 1);
  const double xx = j - c, yy = c - i; /* x to the right, y upwards */
  const double cs = cos(phi_rad), sn = sin(phi_rad);
  const double xs = cs * xx + sn * yy; /* the point that lands on (xx,yy) after turning by +phi */
  const double ys = -sn * xx + cs * yy;
  const double row = c - ys, col = c + xs;
  const double fr = floor(row), fc = floor(col);
  const double ar = row - fr, ac = col - fc;
  int n = 0;
  for (int a = 0; a < 2; ++a)
    for (int b = 0; b < 2; ++b) {
      const int rr = (int)fr + a, cc = (int)fc + b;
      const double wv = (a ? ar : 1.0 - ar) * (b ? ac : 1.0 - ac);
      src[n] = (rr >= 0 && rr < k && cc >= 0 && cc < k) ? rr * k + cc : -1;
      wgt[n] = wv;
      ++n;
    }
}

static void split_angle(double theta_deg, int* s, double* phi_deg) {
  int q = (int)floor(theta_deg / 90.0);
  *s = ((q % 4) + 4) % 4;
  *phi_deg = theta_deg - 90.0 * q;
}

/* First-quadrant filter F_phi of one (co,ci) slice.
 * slices: base[0] (and base[1] = f_y in steerable mode, base[0] = f_x). */
static void first_quadrant_filter(int mode, int k, double phi_deg, const double* b0, const double* b1, double* out) {
  const double phi = phi_deg * ORC_PI / 180.0;
  if (mode == ORC_EXACT90) {
    memcpy(out, b0, sizeof(double) * k * k);
  } else if (mode == ORC_STEERABLE) {
    /* Eq. 17: psi_theta = sin(theta) f_x + cos(theta) f_y */
    for (int t = 0; t < k * k; ++t) out[t] = sin(phi) * b0[t] + cos(phi) * b1[t];
  } else {
    for (int i = 0; i < k; ++i)
      for (int j = 0; j < k; ++j) {
        if (phi_deg == 0.0) { out[i * k + j] = b0[i * k + j]; continue; }
        int src[4]; double wgt[4];
        bilinear_sources(k, phi, i, j, src, wgt);
        double acc = 0.0;
        for (int n = 0; n < 4; ++n)
          if (src[n] >= 0) acc += wgt[n] * b0[src[n]];
        out[i * k + j] = acc;
      }
  }
}

/* Adjoint of first_quadrant_filter: given dF (gradient of F_phi), add the
 * gradient of the base slice(s).  Transposes the linear map above. */
static void first_quadrant_filter_adjoint(int mode, int k, double phi_deg, const double* dF, double* d0, double* d1) {
  const double phi = phi_deg * ORC_PI / 180.0;
  if (mode == ORC_EXACT90) {
    for (int t = 0; t < k * k; ++t) d0[t] += dF[t];
  } else if (mode == ORC_STEERABLE) {
    for (int t = 0; t < k * k; ++t) { d0[t] += sin(phi) * dF[t]; d1[t] += cos(phi) * dF[t]; }
  } else {
    for (int i = 0; i < k; ++i)
      for (int j = 0; j < k; ++j) {
        if (phi_deg == 0.0) { d0[i * k + j] += dF[i * k + j]; continue; }
        int src[4]; double wgt[4];
        bilinear_sources(k, phi, i, j, src, wgt);
        for (int n = 0; n < 4; ++n)
          if (src[n] >= 0) d0[src[n]] += wgt[n] * dF[i * k + j];
      }
  }
}

/* Eq. 5 generalised: materialise the R rotated banks.  Returns 0, or -1 when an
 * exact90 angle is not a multiple of 90 degrees. */
int orc_expand_bank(int mode, int R, const double* angles_deg, int k, int Cout, int Cin,
                    const double* w_base, double* w_rot) {
  const size_t kk = (size_t)k * k, slice_n = (size_t)Cout * Cin;
  double* t0 = (double*)malloc(sizeof(double) * kk);
  double* t1 = (double*)malloc(sizeof(double) * kk);
  int rc = 0;
  for (int r = 0; r < R; ++r) {
    int s; double phi;
    split_angle(angles_deg[r], &s, &phi);
    if (mode == ORC_EXACT90 && phi != 0.0) { rc = -1; break; }
    for (size_t sl = 0; sl < slice_n; ++sl) {
      const double* b0 = w_base + sl * kk;
      const double* b1 = (mode == ORC_STEERABLE) ? w_base + (slice_n + sl) * kk : NULL;
      first_quadrant_filter(mode, k, phi, b0, b1, t0);
      for (int q = 0; q < s; ++q) { rot90_once(t0, t1, k); memcpy(t0, t1, sizeof(double) * kk); }
      memcpy(w_rot + ((size_t)r * slice_n + sl) * kk, t0, sizeof(double) * kk);
    }
  }
  free(t0); free(t1);
  return rc;
}

/* Eq. 16 generalised: dW_base = sum_r  (first-quadrant adjoint)( R_{-r}( dW^(r) ) ). */
int orc_reduce_bank_grad(int mode, int R, const double* angles_deg, int k, int Cout, int Cin,
                         const double* dw_rot, double* dw_base) {
  const size_t kk = (size_t)k * k, slice_n = (size_t)Cout * Cin;
  const int B = (mode == ORC_STEERABLE) ? 2 : 1;
  memset(dw_base, 0, sizeof(double) * B * slice_n * kk);
  double* t0 = (double*)malloc(sizeof(double) * kk);
  double* t1 = (double*)malloc(sizeof(double) * kk);
  int rc = 0;
  for (int r = 0; r < R; ++r) {
    int s; double phi;
    split_angle(angles_deg[r], &s, &phi);
    if (mode == ORC_EXACT90 && phi != 0.0) { rc = -1; break; }
    for (size_t sl = 0; sl < slice_n; ++sl) {
      memcpy(t0, dw_rot + ((size_t)r * slice_n + sl) * kk, sizeof(double) * kk);
      for (int q = 0; q < s; ++q) { rot90_undo_once(t0, t1, k); memcpy(t0, t1, sizeof(double) * kk); }
      double* d0 = dw_base + sl * kk;
      double* d1 = (mode == ORC_STEERABLE) ? dw_base + (slice_n + sl) * kk : NULL;
      first_quadrant_filter_adjoint(mode, k, phi, t0, d0, d1);
    }
  }
  free(t0); free(t1);
  return rc;
}

static inline int out_extent(int H, int k, int stride, int pad) { return (H + 2 * pad - k) / stride + 1; }

/* Eq. 7 (gather form), with zero padding and stride:
 * Y[n,co,r,oy,ox] = sum_ci sum_i sum_j W^(r)[co,ci,i,j] * Xpad[n,ci,oy*s+i-p,ox*s+j-p] */
void orc_rotconv_fwd(const double* x, const double* w_rot, double* y, int N, int Cin, int H, int W, int Cout, int R,
                     int k, int stride, int pad) {
  const int Ho = out_extent(H, k, stride, pad), Wo = out_extent(W, k, stride, pad);
#pragma omp parallel for collapse(3) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int co = 0; co < Cout; ++co)
      for (int r = 0; r < R; ++r)
        for (int oy = 0; oy < Ho; ++oy)
          for (int ox = 0; ox < Wo; ++ox) {
            double acc = 0.0;
            for (int ci = 0; ci < Cin; ++ci)
              for (int i = 0; i < k; ++i) {
                const int h = oy * stride + i - pad;
                if (h < 0 || h >= H) continue;
                for (int j = 0; j < k; ++j) {
                  const int w = ox * stride + j - pad;
                  if (w < 0 || w >= W) continue;
                  acc += w_rot[((((size_t)r * Cout + co) * Cin + ci) * k + i) * k + j] *
                         x[(((size_t)n * Cin + ci) * H + h) * W + w];
                }
              }
            y[((((size_t)n * Cout + co) * R + r) * Ho + oy) * Wo + ox] = acc;
          }
}

/* Same values at a list of sampled outputs: pts[4*t..] = (n, co, oy, ox); all R
 * orientations of each point are returned, out[t*R + r]. */
void orc_rotconv_fwd_at(const double* x, const double* w_rot, const int32_t* pts, int npts, double* out, int N,
                        int Cin, int H, int W, int Cout, int R, int k, int stride, int pad) {
  (void)N;
#pragma omp parallel for schedule(static)
  for (int t = 0; t < npts; ++t) {
    const int n = pts[4 * t], co = pts[4 * t + 1], oy = pts[4 * t + 2], ox = pts[4 * t + 3];
    for (int r = 0; r < R; ++r) {
      double acc = 0.0;
      for (int ci = 0; ci < Cin; ++ci)
        for (int i = 0; i < k; ++i) {
          const int h = oy * stride + i - pad;
          if (h < 0 || h >= H) continue;
          for (int j = 0; j < k; ++j) {
            const int w = ox * stride + j - pad;
            if (w < 0 || w >= W) continue;
            acc += w_rot[((((size_t)r * Cout + co) * Cin + ci) * k + i) * k + j] *
                   x[(((size_t)n * Cin + ci) * H + h) * W + w];
          }
        }
      out[(size_t)t * R + r] = acc;
    }
  }
}

/* Quarter-turn coordinate map used by the scatter formulation: where base tap
 * (m,n) sits inside the filter turned s times, (m',n') = R_s(m,n). */
static void turn_tap(int k, int s, int m, int n, int* mo, int* no) {
  for (int q = 0; q < s; ++q) { const int m2 = k - 1 - n, n2 = m; m = m2; n = n2; }
  *mo = m; *no = n;
}

/* Alg. 1 / Eq. 8 (scatter form), symmetric rotations only (quarter[r] in 0..3),
 * stride 1.  For every input pixel and base tap the channel sum is formed ONCE
 * and added at the R rotated output locations:
 *   Y[co, r, h - m' + p, w - n' + p] += sum_ci X[ci,h,w] * W[co,ci,m,n],  (m',n') = R_r(m,n).
 * Products that land outside the output are dropped. */
void orc_rotconv_fwd_scatter(const double* x, const double* w_base, const int32_t* quarter, double* y, int N, int Cin,
                             int H, int W, int Cout, int R, int k, int pad) {
  const int Ho = out_extent(H, k, 1, pad), Wo = out_extent(W, k, 1, pad);
  memset(y, 0, sizeof(double) * (size_t)N * Cout * R * Ho * Wo);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int co = 0; co < Cout; ++co)
      for (int h = 0; h < H; ++h)
        for (int w = 0; w < W; ++w)
          for (int m = 0; m < k; ++m)
            for (int nn = 0; nn < k; ++nn) {
              double prod = 0.0;
              for (int ci = 0; ci < Cin; ++ci)
                prod += x[(((size_t)n * Cin + ci) * H + h) * W + w] * w_base[(((size_t)co * Cin + ci) * k + m) * k + nn];
              for (int r = 0; r < R; ++r) {
                int mp, np_;
                turn_tap(k, quarter[r], m, nn, &mp, &np_);
                const int oy = h - mp + pad, ox = w - np_ + pad;
                if (oy < 0 || oy >= Ho || ox < 0 || ox >= Wo) continue;
                y[((((size_t)n * Cout + co) * R + r) * Ho + oy) * Wo + ox] += prod;
              }
            }
}

/* Eq. 10 with subgroup pooling (Sec. V-A): group g of filter co holds the
 * orientations r with r mod (R/G) == g; for evenly spaced angles and G = 4
 * these are the four symmetric rotations of one first-quadrant angle.
 * idx = smallest r of the group that attains the maximum. */
void orc_orient_maxpool_fwd(const double* y, double* ypool, uint8_t* idx, int N, int Cout, int R, int G, int Ho, int Wo) {
  const int ng = R / G;
  const size_t P = (size_t)Ho * Wo;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int co = 0; co < Cout; ++co)
      for (int g = 0; g < ng; ++g)
        for (size_t p = 0; p < P; ++p) {
          int best_r = g;
          double best = y[(((size_t)n * Cout + co) * R + g) * P + p];
          for (int r = g + ng; r < R; r += ng) {
            const double v = y[(((size_t)n * Cout + co) * R + r) * P + p];
            if (v > best) { best = v; best_r = r; }
          }
          ypool[(((size_t)n * Cout + co) * ng + g) * P + p] = best;
          idx[(((size_t)n * Cout + co) * ng + g) * P + p] = (uint8_t)best_r;
        }
}

/* Eq. 12: Delta[n,co,r,p] = G[n,co,g,p] * 1[r == idx[n,co,g,p]],  g = r mod (R/G). */
void orc_orient_maxpool_bwd(const double* gpool, const uint8_t* idx, double* dy, int N, int Cout, int R, int G, int Ho,
                            int Wo) {
  const int ng = R / G;
  const size_t P = (size_t)Ho * Wo;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int co = 0; co < Cout; ++co)
      for (int r = 0; r < R; ++r) {
        const int g = r % ng;
        for (size_t p = 0; p < P; ++p) {
          const size_t q = (((size_t)n * Cout + co) * ng + g) * P + p;
          dy[(((size_t)n * Cout + co) * R + r) * P + p] = (idx[q] == r) ? gpool[q] : 0.0;
        }
      }
}

/* Eq. 13 summed over r (Eq. 15), with padding and stride:
 * dX[n,ci,h,w] = sum_r sum_co sum_ij W^(r)[co,ci,i,j] * Delta[n,co,r,(h+p-i)/s,(w+p-j)/s]
 * (terms whose output coordinate is fractional or out of range do not exist). */
void orc_rotconv_bwd_data(const double* dy, const double* w_rot, double* dx, int N, int Cin, int H, int W, int Cout,
                          int R, int k, int stride, int pad) {
  const int Ho = out_extent(H, k, stride, pad), Wo = out_extent(W, k, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int ci = 0; ci < Cin; ++ci)
      for (int h = 0; h < H; ++h)
        for (int w = 0; w < W; ++w) {
          double acc = 0.0;
          for (int r = 0; r < R; ++r)
            for (int co = 0; co < Cout; ++co)
              for (int i = 0; i < k; ++i) {
                const int ty = h + pad - i;
                if (ty < 0 || ty % stride) continue;
                const int oy = ty / stride;
                if (oy >= Ho) continue;
                for (int j = 0; j < k; ++j) {
                  const int tx = w + pad - j;
                  if (tx < 0 || tx % stride) continue;
                  const int ox = tx / stride;
                  if (ox >= Wo) continue;
                  acc += w_rot[((((size_t)r * Cout + co) * Cin + ci) * k + i) * k + j] *
                         dy[((((size_t)n * Cout + co) * R + r) * Ho + oy) * Wo + ox];
                }
              }
          dx[(((size_t)n * Cin + ci) * H + h) * W + w] = acc;
        }
}

/* The same at sampled input positions: pts[4*t..] = (n, ci, h, w). */
void orc_rotconv_bwd_data_at(const double* dy, const double* w_rot, const int32_t* pts, int npts, double* out, int N,
                             int Cin, int H, int W, int Cout, int R, int k, int stride, int pad) {
  (void)N; (void)H; (void)W;
  const int Ho = out_extent(H, k, stride, pad), Wo = out_extent(W, k, stride, pad);
#pragma omp parallel for schedule(static)
  for (int t = 0; t < npts; ++t) {
    const int n = pts[4 * t], ci = pts[4 * t + 1], h = pts[4 * t + 2], w = pts[4 * t + 3];
    double acc = 0.0;
    for (int r = 0; r < R; ++r)
      for (int co = 0; co < Cout; ++co)
        for (int i = 0; i < k; ++i) {
          const int ty = h + pad - i;
          if (ty < 0 || ty % stride) continue;
          const int oy = ty / stride;
          if (oy >= Ho) continue;
          for (int j = 0; j < k; ++j) {
            const int tx = w + pad - j;
            if (tx < 0 || tx % stride) continue;
            const int ox = tx / stride;
            if (ox >= Wo) continue;
            acc += w_rot[((((size_t)r * Cout + co) * Cin + ci) * k + i) * k + j] *
                   dy[((((size_t)n * Cout + co) * R + r) * Ho + oy) * Wo + ox];
          }
        }
    out[t] = acc;
  }
}

/* Eq. 14 summed over the batch, with padding and stride:
 * dW^(r)[co,ci,i,j] = sum_n sum_oy sum_ox Xpad[n,ci,oy*s+i-p,ox*s+j-p] * Delta[n,co,r,oy,ox] */
void orc_rotconv_bwd_weight(const double* x, const double* dy, double* dw_rot, int N, int Cin, int H, int W, int Cout,
                            int R, int k, int stride, int pad) {
  const int Ho = out_extent(H, k, stride, pad), Wo = out_extent(W, k, stride, pad);
#pragma omp parallel for collapse(3) schedule(static)
  for (int r = 0; r < R; ++r)
    for (int co = 0; co < Cout; ++co)
      for (int ci = 0; ci < Cin; ++ci)
        for (int i = 0; i < k; ++i)
          for (int j = 0; j < k; ++j) {
            double acc = 0.0;
            for (int n = 0; n < N; ++n)
              for (int oy = 0; oy < Ho; ++oy) {
                const int h = oy * stride + i - pad;
                if (h < 0 || h >= H) continue;
                for (int ox = 0; ox < Wo; ++ox) {
                  const int w = ox * stride + j - pad;
                  if (w < 0 || w >= W) continue;
                  acc += x[(((size_t)n * Cin + ci) * H + h) * W + w] *
                         dy[((((size_t)n * Cout + co) * R + r) * Ho + oy) * Wo + ox];
                }
              }
            dw_rot[((((size_t)r * Cout + co) * Cin + ci) * k + i) * k + j] = acc;
          }
}

/* Eq. 12 + Eq. 14 at sampled (co,ci) pairs, taking the pooled gradient and idx
 * directly (so the R-fold Delta never has to exist at full size):
 * pairs[2*t..] = (co, ci); out[t][R][k][k]. */
void orc_rotconv_pool_bwd_weight_at(const double* x, const double* gpool, const uint8_t* idx, const int32_t* pairs,
                                    int npairs, double* out, int N, int Cin, int H, int W, int Cout, int R, int G,
                                    int k, int stride, int pad) {
  const int Ho = out_extent(H, k, stride, pad), Wo = out_extent(W, k, stride, pad);
  const int ng = R / G;
#pragma omp parallel for schedule(dynamic)
  for (int t = 0; t < npairs; ++t) {
    const int co = pairs[2 * t], ci = pairs[2 * t + 1];
    double* o = out + (size_t)t * R * k * k;
    for (int q = 0; q < R * k * k; ++q) o[q] = 0.0;
    for (int n = 0; n < N; ++n)
      for (int g = 0; g < ng; ++g)
        for (int oy = 0; oy < Ho; ++oy)
          for (int ox = 0; ox < Wo; ++ox) {
            const size_t q = ((((size_t)n * Cout + co) * ng + g) * Ho + oy) * Wo + ox;
            const int r = idx[q];
            if (r >= R || r % ng != g) continue;   /* Eq. 12: an index that names no member of the group routes nothing */
            const double d = gpool[q];
            for (int i = 0; i < k; ++i) {
              const int h = oy * stride + i - pad;
              if (h < 0 || h >= H) continue;
              for (int j = 0; j < k; ++j) {
                const int w = ox * stride + j - pad;
                if (w < 0 || w >= W) continue;
                o[((size_t)r * k + i) * k + j] += x[(((size_t)n * Cin + ci) * H + h) * W + w] * d;
              }
            }
          }
  }
}
