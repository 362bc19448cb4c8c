// Host side of the fused forward on products of the base bank (kernel: rotconv_p4_fwd_base_kernel.h): bank
// classification against the compiled source patterns, row segments and bands, packing of the base bank, launch.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "rotconv_kernels.h"
#include "rotconv_p4_fwd_base_kernel.h"

namespace rotconv {
namespace {

// base bank -> the LDS image layout [CB][CinPad][9][16] (zero for padded filters / channels)
__global__ __launch_bounds__(256) void k_p4_pack_base(const float* __restrict__ w, float* __restrict__ wt, int CB,
                                                      int CinPad, int Cin, int Cout) {
  const int total = CB * CinPad * 16;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int c16 = e % 16;
  const int ci = (e / 16) % CinPad;
  const int cb = e / (16 * CinPad);
  const int co = cb * 16 + c16;
  const bool in = co < Cout && ci < Cin;
  const float* src = w + (size_t)(in ? co * Cin + ci : 0) * 9;
  float* dst = wt + (size_t)(e / 16) * 144 + c16;
#pragma unroll
  for (int u = 0; u < 9; ++u) dst[u * 16] = in ? src[u] : 0.f;
}

// LDS beside the filter block: the edge arrays, and with `park` banks' second rolling sums parked there 16 bytes per
// bank, quarter turn and thread (eight waves)
size_t base_lds_extra(int park) { return (size_t)2 * 2 * 8 * 144 * 4 + (size_t)park * 4 * 512 * 16; }
bool needs_stream_base(int Cin, int park = 0) { return (size_t)cin_pad_base(Cin) * 576 + base_lds_extra(park) > 160 * 1024; }
// rows a streamed filter block takes: only those the wave chains cover exactly
bool stream_rows_ok(int W) { return (W & 15) == 0 && (W > 128 || (W & (W - 1)) == 0); }
// Banks whose second rolling sum is parked in LDS: three of the four of an R = 16 layer (the benchmark instance then
// keeps 80 instead of 128 sums in registers across the channel loop and no longer spills), when the filter block
// still fits beside them or may be streamed.
int base_park(const rotconv_plan* p) {
  if (p->host.Q != 4) return 0;
  if (!needs_stream_base(p->d.Cin, 3)) return 3;
  if (!needs_stream_base(p->d.Cin, 2)) return 2;      // two banks parked, the filter block still resident
  if (!stream_rows_ok(p->d.W)) return 0;
  return 3;
}

template <int NWX, int NWY, bool FASTW, bool STREAM, int KC, int NQ, int CLS, int PARK>
void launch_i(const P4Geom& g, const float* x, const float* wt, const float* coef, const int32_t* rot_of, float* ov,
              uint8_t* oi, hipStream_t st) {
  const size_t wfl = STREAM ? (size_t)2 * KC * 4 * 144 : (size_t)g.cper * KC * 4 * 144;
  const size_t lds = (wfl + 4 * NWX * NWY * 144) * sizeof(float) + (size_t)PARK * 4 * 64 * NWX * NWY * 16;
  const int grid = (g.units + 7) / 8 * 8;
  auto kern = k_p4_fwd_base<NWX, NWY, FASTW, STREAM, KC, NQ, CLS, PARK>;
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * NWX * NWY), lds, st, x, wt, coef, rot_of, ov, oi, g);
}

template <int NWX, int NWY, int NQ, int CLS, int PARK>
void launch_t(const P4Geom& g, bool fastw, bool stream, const float* x, const float* wt, const float* coef,
              const int32_t* rot_of, float* ov, uint8_t* oi, hipStream_t st) {
  if (g.CinPad == 4) {
    if (fastw) launch_i<NWX, NWY, true, false, 1, NQ, CLS, PARK>(g, x, wt, coef, rot_of, ov, oi, st);
    else launch_i<NWX, NWY, false, false, 1, NQ, CLS, PARK>(g, x, wt, coef, rot_of, ov, oi, st);
  } else if (stream) {
    if (fastw) launch_i<NWX, NWY, true, true, 8, NQ, CLS, PARK>(g, x, wt, coef, rot_of, ov, oi, st);
    else launch_i<NWX, NWY, false, true, 8, NQ, CLS, PARK>(g, x, wt, coef, rot_of, ov, oi, st);
  } else {
    if (fastw) launch_i<NWX, NWY, true, false, 8, NQ, CLS, PARK>(g, x, wt, coef, rot_of, ov, oi, st);
    else launch_i<NWX, NWY, false, false, 8, NQ, CLS, PARK>(g, x, wt, coef, rot_of, ov, oi, st);
  }
}

template <int NQ, int CLS, int PARK>
void launch_c(const P4Geom& g, bool fastw, bool stream, const float* x, const float* wt, const float* coef,
              const int32_t* rot_of, float* ov, uint8_t* oi, hipStream_t st) {
  switch (g.nwx) {
    case 1: launch_t<1, 8, NQ, CLS, PARK>(g, fastw, stream, x, wt, coef, rot_of, ov, oi, st); break;
    case 2: launch_t<2, 4, NQ, CLS, PARK>(g, fastw, stream, x, wt, coef, rot_of, ov, oi, st); break;
    case 4: launch_t<4, 2, NQ, CLS, PARK>(g, fastw, stream, x, wt, coef, rot_of, ov, oi, st); break;
    default: launch_t<8, 1, NQ, CLS, PARK>(g, fastw, stream, x, wt, coef, rot_of, ov, oi, st); break;
  }
}

constexpr int cls_pack(int a, int b = 0, int c = 0, int d = 0) { return a | (b << 2) | (c << 4) | (d << 6); }
// the bank-class lists with a compiled instance
// (a 45 degree bank falls into the lower class: in fp64 its corner taps' source column comes out just below the
// cell boundary; other bank lists run the per-bank kernel)
constexpr int kCls16 = cls_pack(kClsId, kClsLo, kClsLo, kClsHi);     // 0, 22.5, 45, 67.5 degrees (R = 16)
constexpr int kCls8 = cls_pack(kClsId, kClsLo);                      // 0, 45 degrees (R = 8)
constexpr int kClsP4m = cls_pack(kClsId, kClsMirror);                // the filter and its mirror image (p4m, R = 8)

bool cls_compiled(int Q, int cls) {
  return (Q == 4 && cls == kCls16) || (Q == 2 && (cls == kCls8 || cls == kClsP4m));
}

// Row segments of at most 8 waves x 16 product columns; neighbouring segments overlap by 4 pixels on each side (a
// lane at a chain end that is not an image border lacks its neighbour's products and does not store).
int base_geoms(const rotconv_plan* p, P4Geom* out, int max_out) {
  const rotconv_desc& d = p->d;
  P4Geom base{};
  base.N = d.N; base.Cin = d.Cin; base.CinPad = cin_pad_base(d.Cin); base.H = d.H; base.W = d.W;
  base.Cout = d.Cout; base.CB = (d.Cout + 15) / 16; base.R = d.R; base.Q = p->host.Q; base.ng = 1;
  base.out_mode = kOutPooled;
  base.relu = d.activation == ROTCONV_ACT_RELU;
  base.csplit = 1;
  base.cper = base.CinPad == 4 ? 1 : base.CinPad / 32;
  base.nq = p->host.Q;
  int ng = 0, pos = 0;
  while (pos < d.W) {
    int xorg, nwx;
    if (pos == 0) {
      xorg = 0;
      nwx = 1;
      while (nwx * 16 < d.W && nwx < 8) nwx *= 2;
    } else {
      const int need = d.W - (pos - 4);      // product columns from the lane left of `pos` to the border
      nwx = 1;
      while (nwx * 16 < need && nwx < 8) nwx *= 2;
      xorg = nwx * 16 >= need ? d.W - nwx * 16 : pos - 4;    // the last segment ends exactly at the right border
    }
    const int chain_end = xorg + nwx * 16;
    const int hi = chain_end >= d.W ? d.W : chain_end - 4;
    int gi = -1;
    for (int i = 0; i < ng; ++i)
      if (out[i].nwx == nwx && out[i].nseg < 4) gi = i;
    if (gi < 0) {
      if (ng >= max_out) return -1;
      gi = ng++;
      out[gi] = base;
      out[gi].nwx = nwx;
      out[gi].nseg = 0;
      out[gi].inside = 1;
    }
    P4Geom& g = out[gi];
    g.seg_xorg[g.nseg] = xorg; g.seg_lo[g.nseg] = pos; g.seg_hi[g.nseg] = hi;
    if (chain_end > d.W) g.inside = 0;
    g.nseg++;
    pos = hi;
  }
  for (int i = 0; i < ng; ++i) {
    P4Geom& g = out[i];
    const int nwy = 8 / g.nwx;
    long best_cost = -1;
    // rows per band: rounds of workgroups over the 256 CUs x row steps per wave x waves sharing a SIMD
    for (int ty : {1, 2, 4, 8, 16, 32, 64}) {
      const int nbg = (d.H + nwy * ty - 1) / (nwy * ty);
      const long units = (long)d.N * g.CB * nbg * g.nseg;
      const int bands = nbg > 1 ? nwy : std::min(nwy, (d.H + ty - 1) / ty);
      const long cost = ((units + 255) / 256) * (ty + 2) * std::max(4, g.nwx * bands);
      if (best_cost < 0 || cost <= best_cost) { best_cost = cost; g.TY = ty; g.nbg = nbg; g.units = (int)units; }
    }
    g.cost = (int)std::min<long>(best_cost * g.cper, 1L << 30);
  }
  return ng;
}

}  // namespace

// Classes of the plan's banks (two bits per bank) and the coefficients in pattern order [Q][9][4]; -1 when a bank
// fits no class or the plan has more than four banks or several base banks.
int p4_fwd_base_classify(const rotconv_plan* p, std::vector<float>* coef) {
  const int Q = p->host.Q;
  if (p->B != 1 || p->kk != 9 || Q < 2 || Q > 4) return -1;
  if (coef) coef->assign((size_t)Q * 36, 0.f);
  int packed = 0;
  for (int q = 0; q < Q; ++q) {
    int found = -1;
    for (int cls : {kClsId, kClsMirror, kClsLo, kClsHi}) {
      bool ok = true;
      std::vector<float> cf(36, 0.f);
      for (int t = 0; t < 9 && ok; ++t)
        for (int z = 0; z < kMaxNnz && ok; ++z) {
          const int s = p->host.fq_src[(q * 9 + t) * kMaxNnz + z];
          if (s < 0) continue;
          const float cv = p->host.fq_coef[(q * 9 + t) * kMaxNnz + z];
          int slot = -1;
          for (int e = 0; e < 4; ++e)
            if (pat_src(cls, t, e) == s) slot = e;
          if (slot < 0) { ok = false; break; }
          // taps whose coefficient the kernel takes to be one: every tap of a copy, the centre of a turned bank
          if ((cls == kClsId || cls == kClsMirror || t == 4) && cv != 1.0f) { ok = false; break; }
          cf[t * 4 + slot] += cv;
        }
      // a copy must have every tap (a missing one would be read as present)
      if (ok && (cls == kClsId || cls == kClsMirror))
        for (int t = 0; t < 9; ++t) ok = ok && cf[t * 4] == 1.0f;
      if (ok && cf[4 * 4] != 1.0f) ok = false;
      if (ok) {
        found = cls;
        if (coef) std::copy(cf.begin(), cf.end(), coef->begin() + (size_t)q * 36);
        break;
      }
    }
    if (found < 0) return -1;
    packed |= found << (2 * q);
  }
  return packed;
}

// The pooled forward of this plan can run on base products: 3x3 / stride 1 / pad 1, fp32 tensors, ONE pool group
// holding every orientation of a filter, two to four banks with all four quarter turns each and a compiled class
// list, rows the wave chains take (even; multiples of 16 beyond 128 pixels).
bool p4_fwd_base_supported(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  if (d.k != 3 || d.stride != 1 || d.pad != 1 || d.dtype != ROTCONV_F32 || d.pool_op != ROTCONV_POOL_MAX) return false;
  if (p->ng != 1 || p->opt.fwd_base < 0) return false;
  if ((d.W & 1) || (d.W > 128 && (d.W & 15))) return false;
  if ((double)d.Cin * d.H * d.W >= 1073741824.0) return false;     // 32-bit element offsets inside an image
  // a streamed filter block: only rows that the wave chains cover exactly
  if (needs_stream_base(d.Cin) && !stream_rows_ok(d.W)) return false;
  const int Q = p->host.Q;
  for (int i = 0; i < Q * 4; ++i)
    if (p->rot_of[i] < 0) return false;
  const int cls = p4_fwd_base_classify(p, nullptr);
  return cls >= 0 && cls_compiled(Q, cls);
}

size_t p4_fwd_base_pack_floats(const rotconv_plan* p) {
  return (size_t)((p->d.Cout + 15) / 16) * cin_pad_base(p->d.Cin) * 144;
}

void launch_p4_pack_base(const rotconv_plan* p, const float* w, float* wt, hipStream_t st) {
  const int CinPad = cin_pad_base(p->d.Cin), CB = (p->d.Cout + 15) / 16;
  const int total = CB * CinPad * 16;
  hipLaunchKernelGGL(k_p4_pack_base, dim3((total + 255) / 256), dim3(256), 0, st, w, wt, CB, CinPad, p->d.Cin,
                     p->d.Cout);
}

void launch_p4_fwd_base(const rotconv_plan* p, const float* x, const float* wt, float* ypool, uint8_t* idx,
                        hipStream_t st) {
  P4Geom gs[8];
  const int ng = base_geoms(p, gs, 8);
  const int park = base_park(p);
  const bool stream = needs_stream_base(p->d.Cin, park);
  const int cls = p->fwd_base_cls;
  const float* coef = p->dev.fwd_base_coef;
  const int32_t* rot_of = p->dev.rot_of;
  for (int i = 0; i < ng; ++i) {
    const P4Geom& g = gs[i];
    const bool fastw = (p->d.W & 3) == 0 && g.inside;
    if (cls == kCls16 && park == 3) launch_c<4, kCls16, 3>(g, fastw, stream, x, wt, coef, rot_of, ypool, idx, st);
    else if (cls == kCls16 && park == 2) launch_c<4, kCls16, 2>(g, fastw, stream, x, wt, coef, rot_of, ypool, idx, st);
    else if (cls == kCls16) launch_c<4, kCls16, 0>(g, fastw, stream, x, wt, coef, rot_of, ypool, idx, st);
    else if (cls == kCls8) launch_c<2, kCls8, 0>(g, fastw, stream, x, wt, coef, rot_of, ypool, idx, st);
    else launch_c<2, kClsP4m, 0>(g, fastw, stream, x, wt, coef, rot_of, ypool, idx, st);
  }
}

}  // namespace rotconv
