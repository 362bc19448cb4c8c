// Device code of the fused forward of layers whose pool group spans several first-quadrant banks (R = 8, 16 ... orientations
// pooled together, or the eight filters of the p4m group), 3x3 / stride 1 / pad 1, fp32: products of the BASE
// bank only.
//
// Every rotated bank is a linear map of the base filter, W^(q)[t] = sum_u E_q[t][u] w[u] (paper Sec. III-D, Eq. 17;
// the bilinear table of this build; a tap permutation for the mirror image of the p4m group), so its per-tap
// channel contractions are the same linear map of the base bank's nine:
//     P^q_t[co, h, x] = sum_u E_q[t][u] P_u[co, h, x],      P_u = sum_ci w[co,ci,u] X[ci,h,x].
// The matrix cores therefore run ONE conv-equivalent (v_mfma_f32_16x16x4_f32, M = 16 pixels, N = 16 filters,
// K = 4 channels) whatever the number of orientations; the banks' products are formed from the base products on
// the vector ALU (at most four multiply-adds per tap: 0 for the centre, 2 for a corner, 4 for an edge tap of a
// bilinear bank) and placed at their four quarter-turn positions (Eq. 8) exactly as in the single-bank kernel:
//     Y_(q,s)[co, y, x] = sum_t P^q_t[co, y + i_s(t) - 1, x + j_s(t) - 1].
// A lane owns FOUR consecutive pixels of one filter (one accumulator tile per tap), so that the two rolling
// partial sums of all R orientations (2 R registers per pixel) stay in registers beside the products; a wave covers
// 16 pixels x 16 filters of a row and walks down its band.  The maximum over all R orientations and its arg-max
// (Eq. 10) are taken in the lane; nothing R-fold, and no per-bank candidate, reaches memory.
//
// The nnz pattern of E_q is compiled in (a bank is an identity, a mirror image, or a bilinear turn by less /
// more than 45 degrees: the 2 x 2 source cell of every tap is fixed inside each of these classes); the plan's
// table is checked against the pattern when the plan is created and supplies the coefficients.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

#include "rotconv_p4.h"
#include "rotconv_p4_taps.h"

namespace rotconv {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

// How a bank's products follow from the base products.
enum { kClsId = 0, kClsLo = 1, kClsHi = 2, kClsMirror = 3 };
__host__ __device__ constexpr int cls_of(int CLS, int q) { return (CLS >> (2 * q)) & 3; }

__host__ __device__ constexpr int cfloor(double v) {
  const int i = (int)v;
  return v < (double)i ? i - 1 : i;
}
// Source tap e (0..3: the 2 x 2 cell, row-major) of destination tap t for a bank of class cls, or -1.  The bilinear
// classes are represented by 22.5 and 67.5 degrees: inside (0, 45] resp. [45, 90) degrees every tap keeps its cell.
__host__ __device__ constexpr int pat_src(int cls, int t, int e) {
  if (cls == kClsId) return e == 0 ? t : -1;
  if (cls == kClsMirror) return e == 0 ? (t / 3) * 3 + (2 - t % 3) : -1;
  if (t == 4) return e == 0 ? 4 : -1;
  const double c = cls == kClsLo ? 0.9238795325112867 : 0.3826834323650898;
  const double s = cls == kClsLo ? 0.3826834323650898 : 0.9238795325112867;
  const double dr = t / 3 - 1, dc = t % 3 - 1;
  const double rs = 1.0 + c * dr + s * dc, cs = 1.0 - s * dr + c * dc;
  const int rr = cfloor(rs) + e / 2, cc = cfloor(cs) + e % 2;
  return (rr >= 0 && rr < 3 && cc >= 0 && cc < 3) ? rr * 3 + cc : -1;
}

int cin_pad_base(int Cin) { return Cin <= 4 ? 4 : (Cin + 31) / 32 * 32; }

// FASTW:  W % 4 == 0 and no wave chain reaches beyond the row: no load masks, vector stores.
// STREAM: the filter block does not fit LDS: streamed in 32-channel chunks (double buffered).
// KC:     K-steps (of 4 channels) per prefetch chunk: 8, or 1 for layers with at most 4 input channels.
// NQ:     banks; CLS: their classes, two bits each.
// PARK:   banks (the last PARK of them) whose second rolling sum lives in LDS between the row that starts it and the
//         row that continues it, a lane's own slots ([bank][quarter turn][thread] x four pixels): 16 PARK registers
//         less to keep across the channel loop.
template <int NWX, int NWY, bool FASTW, bool STREAM, int KC, int NQ, int CLS, int PARK>
__global__ __launch_bounds__(64 * NWX * NWY) void k_p4_fwd_base(const float* __restrict__ x,
                                                                const float* __restrict__ wt,
                                                                const float* __restrict__ coef,
                                                                const int32_t* __restrict__ rot_of,
                                                                float* __restrict__ out_val,
                                                                uint8_t* __restrict__ out_idx, P4Geom g) {
  constexpr int NW = NWX * NWY;
  constexpr int NT = 64 * NW;
  constexpr int CHF = KC * 4 * 144;      // floats of one chunk of the filter block
  extern __shared__ float smem[];
  float* Wl = smem;                      // resident: [CinPad][9][16]; streamed: [2][32][9][16]
  float* EL = smem + (STREAM ? 2 * CHF : g.cper * CHF);    // [2][NW][9][16] left-edge products of every wave
  float* ER = EL + 2 * NW * 144;         // [2][NW][9][16] right-edge products
  f4* PK = reinterpret_cast<f4*>(ER + 2 * NW * 144) + threadIdx.x;   // [PARK][4][NT] parked sums, this thread's column

  // XCD-aware unit decode: consecutive units (same image rows, different filter blocks) share an XCD's L2.
  const int per_xcd = (g.units + 7) / 8;
  int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (v >= g.units) return;
  const int nchunk = g.CinPad / (4 * KC);
  const int cb = v % g.CB; v /= g.CB;
  const int seg = v % g.nseg; v /= g.nseg;
  const int bg = v % g.nbg;
  const int n = v / g.nbg;

  const int tid = threadIdx.x;
  const float* wsrc = wt + ((size_t)cb * g.CinPad) * 144;
  constexpr int WPT = (CHF / 4 + NT - 1) / NT;   // float4 per thread and chunk when streaming
  f4 wreg[STREAM ? WPT : 1];
  // a staging load = wave-uniform base (filter block, chunk, slot: scalar arithmetic) + the thread's 32-bit byte offset
  const uint32_t tid16 = (uint32_t)tid * 16u;
  auto wload = [&](int c) {
    c = __builtin_amdgcn_readfirstlane(c);
    asm volatile("" : "+s"(c));      // opaque: no per-thread 64-bit addresses kept (and spilled) for a known chunk
#pragma unroll
    for (int k = 0; k < WPT; ++k) {
      const int e = tid + k * NT;
      const char* wk = reinterpret_cast<const char*>(wsrc + (size_t)c * CHF + (size_t)k * NT * 4);
      if (e < CHF / 4) wreg[k] = *reinterpret_cast<const f4*>(wk + tid16);
    }
  };
  auto wstore = [&](int buf) {
#pragma unroll
    for (int k = 0; k < WPT; ++k) {
      const int e = tid + k * NT;
      if (e < CHF / 4) reinterpret_cast<f4*>(Wl + buf * CHF)[e] = wreg[k];
    }
  };
  if (STREAM) {
    wload(0);
    wstore(0);
  } else {
    const f4* src = reinterpret_cast<const f4*>(wsrc);
    f4* dst = reinterpret_cast<f4*>(Wl);
    const int n4 = nchunk * (CHF / 4);
    for (int i = tid; i < n4; i += NT) dst[i] = src[i];
  }
  __syncthreads();

  const int wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64;
  const int wx = wave % NWX, wy = wave / NWX;
  const int lg = lane / 16, lc = lane % 16;
  const int x0 = g.seg_xorg[seg] + wx * 16;
  const int out_lo = g.seg_lo[seg], out_hi = g.seg_hi[seg];
  const int y0 = (bg * NWY + wy) * g.TY;
  const bool live = y0 < g.H;                // else: a band below the image
  const int nsteps = g.TY + 2;
  const int HW = g.H * g.W;

  int rot[NQ * 4];
#pragma unroll
  for (int i = 0; i < NQ * 4; ++i) rot[i] = rot_of[i];

  // A-operand loads: lane (lc, lg) reads X[ci = 4*kstep + lg][h][x0 + lc].  Rows outside the image are loaded from
  // the clamped row and their products discarded; channels beyond Cin meet zero filter taps; pixels beyond W read
  // as zero (only possible without FASTW).
  // The address is the image's base (wave-uniform) plus a 32-bit element offset: row (uniform) + channel + lane pixel
  // (an image has fewer than 2^30 elements: checked when the plan takes this kernel).
  const int pxa = x0 + lc;
  const bool px_ok = pxa < g.W;
  const float* xn = x + (size_t)n * g.Cin * HW;
  const uint32_t lane_px = (uint32_t)(px_ok ? pxa : 0);
  uint32_t lgoff = (uint32_t)lg * (uint32_t)HW;
  asm volatile("" : "+v"(lgoff));   // opaque: keeps the K-step part of the offset scalar
  const uint32_t off_last = (uint32_t)(g.Cin - 1) * (uint32_t)HW;
  auto row_ptr = [&](int t) -> uint32_t {          // element offset of the (clamped) row
    const int h = min(max(y0 - 1 + t, 0), g.H - 1);
    return (uint32_t)h * (uint32_t)g.W;
  };
  auto load_a = [&](uint32_t rp, int kstep) -> float {
    const uint32_t off = min((uint32_t)(kstep * 4) * (uint32_t)HW + lgoff, off_last) + lane_px;
    const float v1 = xn[off + rp];
    if (FASTW) return v1;
    return px_ok ? v1 : 0.f;
  };

  // two rolling partial sums per orientation and pixel
  constexpr int NKEEP = NQ - PARK;       // banks whose second sum stays in registers
  float accA[NQ * 4][4], accB[(NKEEP > 0 ? NKEEP : 1) * 4][4];
#pragma unroll
  for (int r = 0; r < NQ * 4; ++r)
#pragma unroll
    for (int j = 0; j < 4; ++j) accA[r][j] = 0.f;
#pragma unroll
  for (int r = 0; r < NKEEP * 4; ++r)
#pragma unroll
    for (int j = 0; j < 4; ++j) accB[r][j] = 0.f;
#pragma unroll
  for (int r = 0; r < PARK * 4; ++r) PK[r * NT] = f4{0.f, 0.f, 0.f, 0.f};    // read back by this thread only

  float a_cur[KC];
  {
    const uint32_t rp = row_ptr(0);
#pragma unroll
    for (int ks = 0; ks < KC; ++ks) a_cur[ks] = load_a(rp, ks);
    __builtin_amdgcn_s_waitcnt(0x0F70);
  }
  const float* wl_lane = Wl + lg * 144 + lc;
  int seq = 0;                           // chunk steps done (streaming: LDS buffer parity)

  for (int t = 0; t < nsteps; ++t) {
    const int h = y0 - 1 + t;
    const bool row_ok = h >= 0 && h < g.H;
    const uint32_t rp_cur = row_ptr(t);
    const uint32_t rp_nxt = row_ptr(t + 1);
    f4 P[9];

    // One chunk: the MFMAs of its K-steps, each A slot refilled for the next chunk right after its MFMAs, B read
    // from LDS one K-step ahead, behind scheduling fences (the compiler would sink loads to their first use).
    auto chunk = [&](int c, bool first) {
      const bool last = c + 1 == nchunk;
      const uint32_t rp = last ? rp_nxt : rp_cur;
      int kn = (last ? 0 : c + 1) * KC;
      if (KC > 1) asm volatile("" : "+s"(kn));   // opaque: the per-K-step offsets are formed where they are used (a
                                                 // precomputed set per chunk position would be spilled)
      if (STREAM) wload(last ? 0 : c + 1);
      const float* wc = STREAM ? wl_lane + (seq & 1) * CHF : wl_lane + (size_t)c * CHF;
      float bw[2][9];
#pragma unroll
      for (int u = 0; u < 9; ++u) bw[0][u] = wc[u * 16];
#pragma unroll
      for (int ks = 0; ks < KC; ++ks) {
        if (ks + 1 < KC) {
#pragma unroll
          for (int u = 0; u < 9; ++u) bw[(ks + 1) & 1][u] = wc[(ks + 1) * 4 * 144 + u * 16];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 9; ++u) {
          const f4 zero = f4{0.f, 0.f, 0.f, 0.f};
          P[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[ks], bw[ks & 1][u], first && ks == 0 ? zero : P[u], 0, 0, 0);
        }
        a_cur[ks] = load_a(rp, kn + ks);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (STREAM) {
        wstore((seq + 1) & 1);
        __syncthreads();
      }
      ++seq;
    };
    if (live) {
      chunk(0, true);
      for (int c = 1; c < nchunk; ++c) chunk(c, false);
    } else if (STREAM) {
      for (int c = 0; c < nchunk; ++c) {
        wload(c + 1 == nchunk ? 0 : c + 1);
        wstore((seq + 1) & 1);
        __syncthreads();
        ++seq;
      }
    }
    if (!row_ok || !live) {
      asm volatile("" ::: "memory");       // keeps this a branch
#pragma unroll
      for (int u = 0; u < 9; ++u) P[u] = f4{0.f, 0.f, 0.f, 0.f};
    }

    // ---- base products of the neighbouring pixels (all nine taps: a bank's edge taps draw on the centre) ------
    // Lane (lg, lc) holds filter lc, pixels x0 + 4*lg + i, i = 0..3, in P[u][i].
    float nbL[9], nbR[9];
    const int par = t & 1;
    float* el = EL + (par * NW + wave) * 144 + lc;
    float* er = ER + (par * NW + wave) * 144 + lc;
    if (lg == 0) {
#pragma unroll
      for (int u = 0; u < 9; ++u) el[u * 16] = P[u][0];
    }
    if (lg == 3) {
#pragma unroll
      for (int u = 0; u < 9; ++u) er[u * 16] = P[u][3];
    }
    const int addr_up = ((lane + 16) & 63) * 4, addr_dn = ((lane + 48) & 63) * 4;
#pragma unroll
    for (int u = 0; u < 9; ++u) {
      // pinned in VGPRs of their own first (an accumulator element handed straight to the cross-lane read
      // picked the wrong element)
      float first_px = P[u][0], last_px = P[u][3];
      asm volatile("" : "+v"(first_px), "+v"(last_px));
      nbR[u] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(addr_up, __builtin_bit_cast(int, first_px)));
      nbL[u] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(addr_dn, __builtin_bit_cast(int, last_px)));
    }
    __syncthreads();
    if (NWX > 1) {
      const float* eln = EL + (par * NW + wave + 1) * 144 + lc;  // right neighbour's left edge
      const float* erp = ER + (par * NW + wave - 1) * 144 + lc;  // left neighbour's right edge
      const bool at_r = lg == 3, at_l = lg == 0;
      const bool has_r = wx + 1 < NWX, has_l = wx > 0;
#pragma unroll
      for (int u = 0; u < 9; ++u) {
        const float vr = has_r ? eln[u * 16] : 0.f;
        const float vl = has_l ? erp[u * 16] : 0.f;
        nbR[u] = at_r ? vr : nbR[u];
        nbL[u] = at_l ? vl : nbL[u];
      }
    } else {
#pragma unroll
      for (int u = 0; u < 9; ++u) {
        nbR[u] = lg == 3 ? 0.f : nbR[u];
        nbL[u] = lg == 0 ? 0.f : nbL[u];
      }
    }
    // base product of tap u at the lane's pixel jj in -1 .. 4
    auto pe = [&](int u, int jj) -> float { return jj < 0 ? nbL[u] : jj > 3 ? nbR[u] : P[u][jj]; };

    // ---- per bank: its products from the base products, placed at the four quarter-turn positions (Eq. 8),
    //      maximum over its four orientations; then the maximum across the banks (Eq. 10) ------------------------
    const int y = h - 1;                       // output row completed by this step
    const int px0 = x0 + 4 * lg;               // first of this lane's 4 pixels
    const int co = cb * 16 + lc;
    const bool fin = t >= 2 && y < g.H && co < g.Cout && px0 >= out_lo && px0 < out_hi;
    float best[4];
    int besti[4];

    auto bank = [&](auto qc) {
      constexpr int q = decltype(qc)::value;
      constexpr int c = cls_of(CLS, q);
      constexpr bool turned = c == kClsLo || c == kClsHi;
      constexpr bool parked = q >= NKEEP;
      // a parked bank's second sums of the previous row: read at the head of the bank's section, used pixel by pixel
      f4 pB[4];
      f4 nB[4];
      if constexpr (parked) {
#pragma unroll
        for (int s = 0; s < 4; ++s) pB[s] = PK[((q - NKEEP) * 4 + s) * NT];
      }
      // the bank's products of one pixel column jj in -1 .. 4 (a turned bank: up to four multiply-adds per tap)
      auto column = [&](int jj, float (&Cc)[9]) {
        const float* cf = coef + q * 36;
#pragma unroll
        for (int tt = 0; tt < 9; ++tt) {
          if (tt == 4) { Cc[4] = pe(4, jj); continue; }
          float acc = 0.f;
          bool begun = false;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int s = pat_src(c, tt, e);
            if (s < 0) continue;
            const float pv = pe(s, jj);
            acc = begun ? __builtin_fmaf(cf[tt * 4 + e], pv, acc) : cf[tt * 4 + e] * pv;
            begun = true;
          }
          Cc[tt] = acc;
        }
      };
      // a turned bank keeps a sliding window of three columns (j - 1, j, j + 1 in slot (column + 1) % 3): every
      // column is formed once and 27 values are live instead of 54
      float Wn[3][9];
      if constexpr (turned) {
        column(-1, Wn[0]);
        column(0, Wn[1]);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if constexpr (turned) column(j + 1, Wn[(j + 2) % 3]);
        auto val = [&](int tt, int jj) -> float {
          if constexpr (c == kClsId) return pe(tt, jj);
          else if constexpr (c == kClsMirror) return pe((tt / 3) * 3 + (2 - tt % 3), jj);
          else return Wn[(jj + 1) % 3][tt];
        };
        float bv = 0.f;
        int bi = 0;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const int r = q * 4 + s;
          // three taps per filter row; a sum starts from its first term
          float tr[3] = {0.f, 0.f, 0.f};
          bool begun[3] = {false, false, false};
#pragma unroll
          for (int u = 0; u < 9; ++u) {
            const float vv = val(u, j + tap_j(s, u) - 1);
            const int ti = tap_i(s, u);
            tr[ti] = begun[ti] ? tr[ti] + vv : vv;
            begun[ti] = true;
          }
          const float yfin = accA[r][j] + tr[2];   // rows h-2, h-1, h are in: output row h-1 done
          if constexpr (parked) {
            accA[r][j] = pB[s][j] + tr[1];
            nB[s][j] = tr[0];
          } else {
            accA[r][j] = accB[r][j] + tr[1];       // output row h has rows h-1, h
            accB[r][j] = tr[0];                    // output row h+1 has row h
          }
          if (s == 0) {
            bv = yfin;
            bi = rot[r];
          } else {
            // inside a bank the orientation index grows with the quarter turn: the first maximum wins
            const bool gt = yfin > bv;
            bv = gt ? yfin : bv;
            bi = gt ? rot[r] : bi;
          }
        }
        if (q == 0) {
          best[j] = bv;
          besti[j] = bi;
        } else {
          // across banks an equal value wins only with the smaller orientation index (ties: the smallest r)
          const bool take = bv > best[j] || (bv == best[j] && bi < besti[j]);
          best[j] = take ? bv : best[j];
          besti[j] = take ? bi : besti[j];
        }
      }
      if constexpr (parked) {
#pragma unroll
        for (int s = 0; s < 4; ++s) PK[((q - NKEEP) * 4 + s) * NT] = nB[s];
      }
    };
    bank(std::integral_constant<int, 0>{});
    if constexpr (NQ > 1) bank(std::integral_constant<int, 1>{});
    if constexpr (NQ > 2) bank(std::integral_constant<int, 2>{});
    if constexpr (NQ > 3) bank(std::integral_constant<int, 3>{});

    uint32_t pk = 0u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (g.relu) {      // fused ReLU: dead elements get idx 255
        const bool dead = !(best[j] > 0.f);
        best[j] = dead ? 0.f : best[j];
        besti[j] = dead ? 255 : besti[j];
      }
      pk |= (uint32_t)besti[j] << (8 * j);
    }
    if (fin) {
      const size_t off = ((size_t)n * g.Cout + co) * HW + (size_t)y * g.W + px0;
      if (FASTW) {
        *reinterpret_cast<f4*>(out_val + off) = f4{best[0], best[1], best[2], best[3]};
        *reinterpret_cast<uint32_t*>(out_idx + off) = pk;
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (px0 + j < min(g.W, out_hi)) {
            out_val[off + j] = best[j];
            out_idx[off + j] = (uint8_t)(pk >> (8 * j));
          }
      }
    }
  }
}

}  // namespace
}  // namespace rotconv
