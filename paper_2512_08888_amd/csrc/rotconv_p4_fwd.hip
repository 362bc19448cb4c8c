// Fast forward kernel for 3x3, stride 1, pad 1 (fp32): shared-product rotation
// convolution on the fp32 matrix cores (paper Eq. 8, re-designed for CDNA4).
//
// For one first-quadrant bank the nine per-tap channel contractions
//     P_u[co, h, x] = sum_ci F[co,ci,u] * X[ci,h,x]           (u = base tap)
// are formed ONCE with v_mfma_f32_16x16x4_f32 (M = 16 pixels, N = 16 filters,
// K = 4 input channels) and then placed at the four quarter-turn positions
//     Y_s[co, y, x] = sum_u P_u[co, y + i_s(u) - 1, x + j_s(u) - 1],  (i_s,j_s) = R_s(u)
// entirely in registers: a wave owns 16 filters x 32 consecutive pixels of one
// image row and walks down the rows of its band, so a row of P feeds the output
// rows above, at and below it through two rolling partial sums per rotation;
// column shifts are register renames (each lane holds 8 consecutive pixels),
// with the one neighbouring value per side fetched from the adjacent lane group
// (ds_bpermute) or the adjacent wave (a few words of LDS per row).  The max over
// the bank's rotations and its arg-max are taken in registers and stored once.
// Nothing R-fold ever reaches memory, and the input row is read once per bank.
//
// The filter block (16 filters x all input channels x 9 taps) stays resident in
// LDS for the life of the workgroup when it fits (Cin <= 224); deeper inputs
// stream it through two 32-channel LDS buffers, one barrier per chunk.  Input
// rows go straight from global memory into the A-operand registers (8-byte
// loads, 128 B contiguous per 16 lanes), each slot refilled one chunk ahead;
// scheduling fences keep those loads and the LDS reads of the B operand where
// they are issued (the compiler would otherwise sink them to their first use).
//
// Rows wider than the 256 pixels a workgroup's eight waves can chain are cut
// into segments that overlap by 8 pixels (the products of the overlap are
// recomputed, about 6 % at W = 512); a segment writes only the pixels whose
// both neighbours it holds.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>

#include "rotconv_bf16.h"
#include "rotconv_kernels.h"
#include "rotconv_p4.h"
#include "rotconv_p4_taps.h"

namespace rotconv {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

// KC (template parameter): K-steps (of 4 channels) per prefetch chunk: 8 (channels padded to 32), or 1 for layers
// with at most 4 input channels (a network's first layer: channels padded to 4, an eighth of the matrix work)
int cin_pad_f32(int Cin) { return Cin <= 4 ? 4 : (Cin + 31) / 32 * 32; }

// UNPOOLED: write every orientation (rotconv_fwd); else max + arg-max over the bank's rotations.
// FASTW:    W % 8 == 0 and no wave chain reaches beyond the row: no load masks, vector stores.
// STREAM:   the filter block does not fit LDS: stream it in 32-channel chunks.
// NQ: banks folded into the 16 filter columns of a wave (1, 2 or 4).  NQ > 1 serves a pool group that spans all NQ
//     banks of the plan (R = 4 NQ orientations pooled together): column n holds bank n / (16/NQ), filter n % (16/NQ);
//     every lane places and maximises its own bank's four rotations and the maximum across the banks is a
//     rotate-and-compare inside the 16-lane row (DPP), so no per-bank candidates go through memory.
template <int NWX, int NWY, bool UNPOOLED, bool FASTW, bool STREAM, int KC, int NQ>
__global__ __launch_bounds__(64 * NWX * NWY) void k_p4_fwd(const float* __restrict__ x, const float* __restrict__ wt,
                                                           const int32_t* __restrict__ rot_of,
                                                           float* __restrict__ out_val, uint8_t* __restrict__ out_idx,
                                                           P4Geom g) {
  constexpr int NW = NWX * NWY;
  constexpr int NT = 64 * NW;
  constexpr int CHF = KC * 4 * 144;      // floats of one 32-channel chunk of the filter block
  extern __shared__ float smem[];
  float* Wl = smem;                      // resident: [CinPad][9][16]; streamed: [2][32][9][16]
  float* EL = smem + (STREAM ? 2 * CHF : g.cper * CHF);    // [2][NW][8][16] left-edge values of every wave
  float* ER = EL + 2 * NW * 128;         // [2][NW][8][16] right-edge values

  // XCD-aware unit decode: consecutive units (same image rows, different filter
  // blocks / banks) go to the same XCD so they share its L2 copy of the input.
  const int per_xcd = (g.units + 7) / 8;
  int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (v >= g.units) return;
  // Channel split (small maps with deep inputs): the workgroup contracts the 32-channel chunks [c_lo, c_hi) only and
  // writes its unpooled sums into part `sp`; the parts are added in order afterwards.  Without a split: all chunks.
  const int sp = v % g.csplit; v /= g.csplit;
  const int nchunk = g.CinPad / (4 * KC);
  const int c_lo = sp * g.cper, c_hi = min(nchunk, c_lo + g.cper);
  const int cb = v % g.CB; v /= g.CB;
  const int q = v % g.Q; v /= g.Q;
  const int seg = v % g.nseg; v /= g.nseg;
  const int bg = v % g.nbg;
  const int n = v / g.nbg;

  const int tid = threadIdx.x;
  const float* wsrc = wt + ((size_t)(q * g.CB + cb) * g.CinPad) * 144;
  constexpr int WPT = (CHF / 4 + NT - 1) / NT;   // float4 per thread and chunk when streaming
  f4 wreg[STREAM ? WPT : 1];
  auto wload = [&](int c) {
#pragma unroll
    for (int k = 0; k < WPT; ++k) {
      const int e = tid + k * NT;
      if (e < CHF / 4) wreg[k] = reinterpret_cast<const f4*>(wsrc + (size_t)c * CHF)[e];
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
  } else if (g.raw_w) {
    // wt is the caller's w[Cout][Cin][9]: the block's sixteen filters at one (channel, tap) are sixteen loads 9 Cin
    // floats apart (consecutive lanes: consecutive addresses) and one 64-byte row of the block; zeros beyond Cout / Cin
    const int pairs = (c_hi - c_lo) * (CHF / 16), e_lo = c_lo * (CHF / 16), e_end = g.Cin * 9;
    const float* wrow = wt + (size_t)cb * 16 * e_end;
    for (int i = tid; i < pairs; i += NT) {
      const int e = e_lo + i;                    // ci * 9 + u
      f4 v[4];
#pragma unroll
      for (int f = 0; f < 16; ++f)
        v[f / 4][f % 4] = (e < e_end && cb * 16 + f < g.Cout) ? wrow[(size_t)f * e_end + e] : 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) reinterpret_cast<f4*>(Wl)[i * 4 + k] = v[k];
    }
  } else {
    const f4* src = reinterpret_cast<const f4*>(wsrc + (size_t)c_lo * CHF);
    f4* dst = reinterpret_cast<f4*>(Wl);
    const int n4 = (c_hi - c_lo) * (CHF / 4);
    for (int i = tid; i < n4; i += NT) dst[i] = src[i];
  }
  __syncthreads();

  // the wave index as a scalar: everything derived from it (band, rows, validity) is wave-uniform and the
  // compiler can branch on it without masking lanes
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64;
  const int wx = wave % NWX, wy = wave / NWX;
  const int lg = lane / 16, lc = lane % 16;
  const int x0 = g.seg_xorg[seg] + wx * 32;
  const int out_lo = g.seg_lo[seg], out_hi = g.seg_hi[seg];
  const int y0 = (bg * NWY + wy) * g.TY;
  const bool live = y0 < g.H;                // else: a band below the image
  const int nsteps = g.TY + 2;
  const int HW = g.H * g.W;

  constexpr int FPB = 16 / NQ;               // filters per wave
  const int qi = NQ > 1 ? lc / FPB : q;       // this lane's bank
  int rot[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) rot[s] = rot_of[qi * 4 + s];

  // A-operand loads: lane (lc, lg) reads X[ci = 4*kstep + lg][h][x0 + 2*lc .. +1].  The address is a
  // per-row lane pointer plus a 32-bit channel offset.  Products of rows outside the image are discarded,
  // channels beyond Cin meet zero filter taps, so both only need a valid address; pixels beyond W must
  // read as zero (only possible when W % 32 != 0).
  const int pxa = x0 + 2 * lc;
  const bool px_ok = pxa < g.W;
  const float* xn = x + (size_t)n * g.Cin * HW + (px_ok ? pxa : 0);
  uint32_t lgoff = (uint32_t)lg * (uint32_t)HW;
  asm volatile("" : "+v"(lgoff));   // opaque: keeps the K-step part of the offset scalar (no per-load vector multiply)
  const uint32_t off_last = (uint32_t)(g.Cin - 1) * (uint32_t)HW;   // channels beyond Cin read channel Cin-1
  auto row_ptr = [&](int t) -> const float* {
    const int h = min(max(y0 - 1 + t, 0), g.H - 1);
    return xn + (size_t)h * g.W;
  };
  auto load_a = [&](const float* rp, int kstep) -> float2 {
    const uint32_t off = min((uint32_t)(kstep * 4) * (uint32_t)HW + lgoff, off_last);
    const float2 v2 = *reinterpret_cast<const float2*>(rp + off);
    if (FASTW) return v2;
    return px_ok ? v2 : make_float2(0.f, 0.f);
  };

  float accA[4][8], accB[4][8];
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int j = 0; j < 8; ++j) { accA[s][j] = 0.f; accB[s][j] = 0.f; }

  // A operands of one 32-channel chunk; each slot is refilled for the next chunk (possibly of the
  // next row) right after its MFMAs have been issued, so the prefetch distance is one chunk.
  float2 a_cur[KC];
  {
    const float* rp = row_ptr(0);
#pragma unroll
    for (int ks = 0; ks < KC; ++ks) a_cur[ks] = load_a(rp, c_lo * KC + ks);
    __builtin_amdgcn_s_waitcnt(0x0F70);
  }
  const float* wl_lane = Wl + lg * 144 + lc;
  int seq = 0;                           // chunk steps done (streaming: LDS buffer parity)

  for (int t = 0; t < nsteps; ++t) {
    const int h = y0 - 1 + t;
    const bool row_ok = h >= 0 && h < g.H;
    const float* rp_cur = row_ptr(t);
    const float* rp_nxt = row_ptr(t + 1);
    f4 P[9][2];   // written by the row's first K-step (accumulator input = constant zero), or zeroed below

    // One 32-channel chunk: MFMAs of its eight K-steps, each slot of A refilled for the next chunk right
    // after its MFMAs, B read from LDS one K-step ahead.  The scheduling fences keep loads and LDS reads
    // where they are issued; left alone the compiler sinks them next to their first use and waits there.
    auto chunk = [&](int c, bool first) {
      const bool last = c + 1 == c_hi;
      const float* rp = last ? rp_nxt : rp_cur;
      const int kn = (last ? c_lo : c + 1) * KC;
      if (STREAM) wload(last ? 0 : c + 1);         // streamed blocks are never split: c_lo = 0
      const float* wc = STREAM ? wl_lane + (seq & 1) * CHF : wl_lane + (size_t)(c - c_lo) * CHF;
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
          P[u][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[ks].x, bw[ks & 1][u], first && ks == 0 ? zero : P[u][0], 0, 0, 0);
          P[u][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[ks].y, bw[ks & 1][u], first && ks == 0 ? zero : P[u][1], 0, 0, 0);
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
    // A row above / below the image (first and last band only) is multiplied like any other, from the clamped
    // row's values, and its products are then discarded: zeroing them ahead of the branch instead would put
    // 72 register moves on every row's path.  A wave whose whole band lies below the image (the workgroup's bands
    // need not divide H) multiplies nothing: it only keeps the workgroup's barriers and filter stages in step.
    if (live) {
      chunk(c_lo, true);
      for (int c = c_lo + 1; c < c_hi; ++c) chunk(c, false);
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
      for (int u = 0; u < 9; ++u) { P[u][0] = f4{0.f, 0.f, 0.f, 0.f}; P[u][1] = f4{0.f, 0.f, 0.f, 0.f}; }
    }

    // ---- neighbour values across lane groups and waves --------------------------
    // Lane (lg, lc) holds filter lc, pixels x0 + 8*lg + j, j = 2*i + b for P[u][b][i].
    float nbL[9], nbR[9];  // P_u at pixel (first - 1) resp. (last + 1) of this lane's 8 pixels
    const int par = t & 1;
    float* el = EL + (par * NW + wave) * 128 + lc;
    float* er = ER + (par * NW + wave) * 128 + lc;
    if (lg == 0) {
#pragma unroll
      for (int u = 0; u < 9; ++u)
        if (u != 4) el[edge_slot(u) * 16] = P[u][0][0];
    }
    if (lg == 3) {
#pragma unroll
      for (int u = 0; u < 9; ++u)
        if (u != 4) er[edge_slot(u) * 16] = P[u][1][3];
    }
    const int addr_up = ((lane + 16) & 63) * 4, addr_dn = ((lane + 48) & 63) * 4;
#pragma unroll
    for (int u = 0; u < 9; ++u) {
      if (u == 4) { nbL[u] = 0.f; nbR[u] = 0.f; continue; }
      // The sources are pinned in VGPRs of their own first: handing an element of the
      // accumulator vector straight to the cross-lane read picked the wrong element.
      float first_px = P[u][0][0], last_px = P[u][1][3];
      asm volatile("" : "+v"(first_px), "+v"(last_px));
      nbR[u] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(addr_up, __builtin_bit_cast(int, first_px)));
      nbL[u] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(addr_dn, __builtin_bit_cast(int, last_px)));
    }
    __syncthreads();
    if (NWX > 1) {
      // all lanes read both neighbour-wave slots (in bounds for every wave), then select; a chain
      // end has no neighbour: zero, which is right at an image border (other ends are not stored)
      const float* eln = EL + (par * NW + wave + 1) * 128 + lc;  // right neighbour's left edge
      const float* erp = ER + (par * NW + wave - 1) * 128 + lc;  // left neighbour's right edge
      const bool at_r = lg == 3, at_l = lg == 0;
      const bool has_r = wx + 1 < NWX, has_l = wx > 0;
#pragma unroll
      for (int u = 0; u < 9; ++u) {
        if (u == 4) continue;
        const float vr = has_r ? eln[edge_slot(u) * 16] : 0.f;
        const float vl = has_l ? erp[edge_slot(u) * 16] : 0.f;
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

    // ---- place the row of products at the rotated positions (Eq. 8) --------------
    const int y = h - 1;                       // output row completed by this step
    const int px0 = x0 + 8 * lg;               // first of this lane's 8 pixels
    const int co = NQ > 1 ? cb * FPB + lc % FPB : cb * 16 + lc;
    const bool fin = t >= 2 && y < g.H && co < g.Cout && px0 >= out_lo && px0 < out_hi && (NQ == 1 || lc < FPB);
    float best[8];
    uint32_t pk[2] = {0u, 0u};                 // arg-max bytes of the lane's 8 pixels
    int grp_r = 0;                             // any rotation of the bank (its pool group)
    bool first = true;
    auto place = [&](int s, int j, float& yfin) {
      // three taps per filter row; a sum starts from its first term (0 + v is an instruction: it is not v for v = -0)
      float tr[3] = {0.f, 0.f, 0.f};
      bool begun[3] = {false, false, false};
#pragma unroll
      for (int u = 0; u < 9; ++u) {
        const int jj = j + tap_j(s, u) - 1;
        const float val = jj < 0 ? nbL[u] : jj > 7 ? nbR[u] : P[u][jj & 1][jj >> 1];
        const int ti = tap_i(s, u);
        tr[ti] = begun[ti] ? tr[ti] + val : val;
        begun[ti] = true;
      }
      const float t0 = tr[0], t1 = tr[1], t2 = tr[2];
      yfin = accA[s][j] + t2;         // rows h-2, h-1, h are in: output row h-1 done
      accA[s][j] = accB[s][j] + t1;   // output row h has rows h-1, h
      accB[s][j] = t0;                // output row h+1 has row h
    };
    if (UNPOOLED) {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        float yfin[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) place(s, j, yfin[j]);
        if (fin && rot[s] >= 0) {
          float* o = out_val + ((((size_t)sp * g.N + n) * g.Cout + co) * g.R + rot[s]) * HW + (size_t)y * g.W + px0;
          if (FASTW) {
            reinterpret_cast<f4*>(o)[0] = f4{yfin[0], yfin[1], yfin[2], yfin[3]};
            reinterpret_cast<f4*>(o)[1] = f4{yfin[4], yfin[5], yfin[6], yfin[7]};
          } else {
#pragma unroll
            for (int j = 0; j < 8; ++j)
              if (px0 + j < min(g.W, out_hi)) o[j] = yfin[j];
          }
        }
      }
    } else {
      // pixel by pixel: the four rotations' values, their max and arg-max (smallest r wins ties)
      if (NQ == 1) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
          if (rot[s] >= 0) { grp_r = rot[s]; first = false; }
      } else {
        first = false;      // all rotations present, one pool group (channel = co)
      }
      // all four quarter turns in the orientation set (every closed set; wave-uniform): plain compare chain
      const bool allrot = NQ > 1 || (rot[0] | rot[1] | rot[2] | rot[3]) >= 0;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float bv = 0.f;
        int bi = 0;
        float yv[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) place(s, j, yv[s]);
        if (allrot) {
          bv = yv[0];
          bi = rot[0];
#pragma unroll
          for (int s = 1; s < 4; ++s) {
            const bool gt = yv[s] > bv;
            bv = gt ? yv[s] : bv;
            bi = gt ? rot[s] : bi;
          }
        } else {
          bool have = false;
#pragma unroll
          for (int s = 0; s < 4; ++s) {
            if (rot[s] >= 0) {
              const bool gt = !have || yv[s] > bv;
              bv = gt ? yv[s] : bv;
              bi = gt ? rot[s] : bi;
              have = true;
            }
          }
        }
        if (NQ > 1) {
          // maximum across the banks: the lanes of one filter sit FPB apart inside the 16-lane row
          auto other = [&](int ov_bits, int oi) {
            const float ov = __builtin_bit_cast(float, ov_bits);
            const bool take = ov > bv || (ov == bv && oi < bi);     // ties: the smallest orientation index
            bv = take ? ov : bv;
            bi = take ? oi : bi;
          };
          other(__builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, bv), 0x128, 0xf, 0xf, false),
                __builtin_amdgcn_update_dpp(0, bi, 0x128, 0xf, 0xf, false));                       // row_ror:8
          if (NQ == 4)
            other(__builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, bv), 0x124, 0xf, 0xf, false),
                  __builtin_amdgcn_update_dpp(0, bi, 0x124, 0xf, 0xf, false));                     // row_ror:4
        }
        best[j] = bv;
        pk[j >> 2] |= (uint32_t)bi << (8 * (j & 3));
      }
    }
    if (!UNPOOLED && g.relu) {      // fused ReLU (pooled output only): dead elements get idx 255
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const bool dead = !(best[j] > 0.f);
        best[j] = dead ? 0.f : best[j];
        pk[j >> 2] |= dead ? 0xffu << (8 * (j & 3)) : 0u;
      }
    }
    if (!UNPOOLED && fin && !first) {
      size_t chan;
      if (g.out_mode == kOutPooled) {
        // every rotation of this bank lies in pool group (r mod ng); pooled channel = co*ng + group
        chan = (size_t)n * g.Cout * g.ng + (size_t)co * g.ng + (grp_r % g.ng);
      } else {  // kOutPartial: per-bank candidates [Q][N][Cout][H][W]
        chan = ((size_t)q * g.N + n) * g.Cout + co;
      }
      const size_t off = chan * HW + (size_t)y * g.W + px0;
      if (FASTW) {
        f4* o = reinterpret_cast<f4*>(out_val + off);
        o[0] = f4{best[0], best[1], best[2], best[3]};
        o[1] = f4{best[4], best[5], best[6], best[7]};
        *reinterpret_cast<uint2*>(out_idx + off) = make_uint2(pk[0], pk[1]);
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (px0 + j < min(g.W, out_hi)) {
            out_val[off + j] = best[j];
            out_idx[off + j] = (uint8_t)(pk[j >> 2] >> (8 * (j & 3)));
          }
      }
    }
  }
}

// Max over the per-bank candidates of a pool group that spans several banks.
// Candidates [Q][N][Cout][HW]; group g of filter co collects banks q with (r mod ng) == g.
__global__ __launch_bounds__(256) void k_p4_combine(const float* __restrict__ pv, const uint8_t* __restrict__ pi,
                                                    const int32_t* __restrict__ rot_of, float* __restrict__ ypool,
                                                    uint8_t* __restrict__ idx, int N, int Cout, int HW, int Q, int ng,
                                                    int relu) {
  const int p = blockIdx.x * 256 + threadIdx.x;
  if (p >= HW) return;
  const int chan = blockIdx.y, n = blockIdx.z;  // chan = co*ng + grp
  const int co = chan / ng, grp = chan % ng;
  float best = 0.f;
  int bi = 255;
  for (int q = 0; q < Q; ++q) {
    int r0 = -1;
    for (int s = 0; s < 4; ++s)
      if (rot_of[q * 4 + s] >= 0) { r0 = rot_of[q * 4 + s]; break; }
    if (r0 < 0 || r0 % ng != grp) continue;
    const size_t o = (((size_t)q * N + n) * Cout + co) * HW + p;
    const float vq = pv[o];
    const int iq = pi[o];
    if (bi == 255 || vq > best || (vq == best && iq < bi)) { best = vq; bi = iq; }
  }
  const size_t o = ((size_t)n * Cout * ng + chan) * HW + p;
  const bool dead = relu && !(best > 0.f);
  ypool[o] = dead ? 0.f : best;
  idx[o] = dead ? (uint8_t)255 : (uint8_t)bi;
}

// Channel split: y = sum of the parts, ascending (four elements per thread, scalar tail).
__global__ __launch_bounds__(256) void k_p4_sum_parts(const float* __restrict__ part, float* __restrict__ y,
                                                      size_t n_elem, int nparts) {
  const size_t n4 = n_elem / 4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
    f4 a = reinterpret_cast<const f4*>(part)[i];
    for (int k = 1; k < nparts; ++k) a += reinterpret_cast<const f4*>(part + (size_t)k * n_elem)[i];
    reinterpret_cast<f4*>(y)[i] = a;
  }
  for (size_t e = n4 * 4 + (size_t)blockIdx.x * 256 + threadIdx.x; e < n_elem; e += (size_t)gridDim.x * 256) {
    float v = part[e];
    for (int k = 1; k < nparts; ++k) v += part[(size_t)k * n_elem + e];
    y[e] = v;
  }
}

// Channel split, pooled: every orientation's sum over the parts (ascending), then max / arg-max over the pool
// group (first maximum wins) and the fused activation.  One thread per pooled element.
__global__ __launch_bounds__(256) void k_p4_sum_pool(const float* __restrict__ part, float* __restrict__ ypool,
                                                     uint8_t* __restrict__ idx, size_t n_elem, int nparts, int NC,
                                                     int R, int ng, int HW, int relu) {
  const size_t total = (size_t)NC * ng * HW;       // NC = N * Cout
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int px = (int)(e % HW);
  const int grp = (int)((e / HW) % ng);
  const size_t nc = e / ((size_t)HW * ng);
  const float* yb = part + nc * R * HW + px;
  float best = 0.f;
  int bi = -1;
  for (int r = grp; r < R; r += ng) {
    float v = yb[(size_t)r * HW];
    for (int k = 1; k < nparts; ++k) v += yb[(size_t)k * n_elem + (size_t)r * HW];
    if (bi < 0 || v > best) { best = v; bi = r; }
  }
  const bool dead = relu && !(best > 0.f);
  ypool[e] = dead ? 0.f : best;
  idx[e] = dead ? (uint8_t)255 : (uint8_t)bi;
}

// base bank(s) -> Q first-quadrant banks in the LDS image layout [Q][CB][CinPad][9][16]
// (zero for padded filters / channels).
__global__ __launch_bounds__(256) void k_p4_pack_fwd(const float* __restrict__ w, float* __restrict__ wt,
                                                     const int32_t* __restrict__ fq_src,
                                                     const float* __restrict__ fq_coef,
                                                     const double* __restrict__ fq_coef64, int Q, int CB, int CinPad,
                                                     int Cin, int Cout, int round16, int nq) {
  // nq > 1: the banks are folded into the 16 columns (column n = bank n / (16/nq), filter n % (16/nq)): [CB'][CinPad]...
  // One thread per (bank, filter, channel): its nine taps read the same 36 bytes of w.
  const int total = (nq > 1 ? 1 : Q) * CB * CinPad * 16;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int c16 = e % 16;
  const int ci = (e / 16) % CinPad;
  const int cb = (e / (16 * CinPad)) % CB;
  const int fpb = 16 / nq;
  const int q = nq > 1 ? c16 / fpb : e / (16 * CinPad * CB);
  const int co = nq > 1 ? cb * fpb + c16 % fpb : cb * 16 + c16;
  const bool in = co < Cout && ci < Cin;
  const int slices = Cout * Cin;
  const float* src = w + (size_t)(in ? co * Cin + ci : 0) * 9;
  float* dst = wt + (size_t)(e / 16) * 144 + c16;
#pragma unroll
  for (int u = 0; u < 9; ++u) {
    float acc = 0.f;
    if (round16) {    // bf16 plans: the combination in fp64, rounded to fp32 and to bf16 once each
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
    dst[u * 16] = acc;
  }
}

template <int NWX, int NWY, bool UNPOOLED, bool FASTW, bool STREAM, int KC = 8, int NQ = 1>
void launch_i(const P4Geom& g, const float* x, const float* wt, const int32_t* rot_of, float* ov, uint8_t* oi,
              hipStream_t st) {
  const size_t wfl = STREAM ? (size_t)2 * KC * 4 * 144 : (size_t)g.cper * KC * 4 * 144;
  const size_t lds = (wfl + 4 * NWX * NWY * 128) * sizeof(float);
  const int grid = (g.units + 7) / 8 * 8;
  auto kern = k_p4_fwd<NWX, NWY, UNPOOLED, FASTW, STREAM, KC, NQ>;
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * NWX * NWY), lds, st, x, wt, rot_of, ov, oi, g);
}

template <int NWX, int NWY>
void launch_t(const P4Geom& g, bool fastw, bool stream, const float* x, const float* wt, const int32_t* rot_of,
              float* ov, uint8_t* oi, hipStream_t st) {
  const bool unp = g.out_mode == kOutUnpooled;
  if (g.nq > 1) {           // banks folded into the columns: pooled output, whole K chunks; a streamed block only
                            // for rows without overhang (p4_fwd_fold sees to that)
    if (g.nq == 4) {
      if (stream) launch_i<NWX, NWY, false, true, true, 8, 4>(g, x, wt, rot_of, ov, oi, st);
      else if (fastw) launch_i<NWX, NWY, false, true, false, 8, 4>(g, x, wt, rot_of, ov, oi, st);
      else launch_i<NWX, NWY, false, false, false, 8, 4>(g, x, wt, rot_of, ov, oi, st);
    } else {
      if (stream) launch_i<NWX, NWY, false, true, true, 8, 2>(g, x, wt, rot_of, ov, oi, st);
      else if (fastw) launch_i<NWX, NWY, false, true, false, 8, 2>(g, x, wt, rot_of, ov, oi, st);
      else launch_i<NWX, NWY, false, false, false, 8, 2>(g, x, wt, rot_of, ov, oi, st);
    }
    return;
  }
  if (g.CinPad == 4) {      // at most 4 input channels: one K-step per row
    if (unp && fastw) launch_i<NWX, NWY, true, true, false, 1>(g, x, wt, rot_of, ov, oi, st);
    else if (unp) launch_i<NWX, NWY, true, false, false, 1>(g, x, wt, rot_of, ov, oi, st);
    else if (fastw) launch_i<NWX, NWY, false, true, false, 1>(g, x, wt, rot_of, ov, oi, st);
    else launch_i<NWX, NWY, false, false, false, 1>(g, x, wt, rot_of, ov, oi, st);
    return;
  }
  if (unp) {
    if (stream) launch_i<NWX, NWY, true, false, true>(g, x, wt, rot_of, ov, oi, st);   // deep inputs: streamed block
    else if (fastw) launch_i<NWX, NWY, true, true, false>(g, x, wt, rot_of, ov, oi, st);
    else launch_i<NWX, NWY, true, false, false>(g, x, wt, rot_of, ov, oi, st);
  } else if (stream) {
    if (fastw) launch_i<NWX, NWY, false, true, true>(g, x, wt, rot_of, ov, oi, st);
    else launch_i<NWX, NWY, false, false, true>(g, x, wt, rot_of, ov, oi, st);   // a wave chain overhangs the row
  } else if (fastw) {
    launch_i<NWX, NWY, false, true, false>(g, x, wt, rot_of, ov, oi, st);
  } else {
    launch_i<NWX, NWY, false, false, false>(g, x, wt, rot_of, ov, oi, st);
  }
}

// Is the filter block of 16 filters too large to stay in LDS next to the edge arrays?
bool needs_stream(int Cin) {
  return (size_t)cin_pad_f32(Cin) * 576 + 16384 > 160 * 1024;
}

}  // namespace

bool p4_fwd_supported(const rotconv_plan* p) {
  const rotconv_desc& d = p->d;
  if (d.k != 3 || d.stride != 1 || d.pad != 1) return false;   // bf16 plans run these kernels on widened copies
  if (d.W & 1) return false;
  if (d.W > 256 && (d.W & 31)) return false;          // segmented rows need whole-lane validity
  // the streaming variant is built for W % 32 == 0; narrower maps split the channels instead
  if (needs_stream(d.Cin) && (d.W & 31) && p4_fwd_csplit(p, false) < 2) return false;
  return true;
}

namespace {
// Cost of a launch plan in quarter row steps (a wave's 144 matrix instructions of one 32-channel chunk and row,
// about 2 us, count 4): the sum of its launches' band costs.
long plan_cost(const rotconv_plan* p, int out_mode, int csplit, int nq) {
  P4Geom gs[4];
  const int n = p4_fwd_geoms(p, out_mode, gs, 4, csplit, nq);
  if (n < 0) return -1;
  long c = 0;
  for (int i = 0; i < n; ++i) c += gs[i].cost;
  return c;
}
}  // namespace

// Parts the channel contraction is split into (1: no split).  Small maps with deep inputs give the (filter block,
// band) decomposition too few workgroups, each with a long serial contraction; splitting the 32-channel chunks over
// workgroups (at most 7 chunks each, so the filter share stays LDS-resident) costs one unpooled fp32 part per split
// and an ordered sum.  `pooled`: the caller wants the pooled output (the alternative is the fused pooled kernel,
// with the banks folded where the plan allows it).
int p4_fwd_csplit(const rotconv_plan* p, bool pooled) {
  const rotconv_desc& d = p->d;
  const int CinPad = cin_pad_f32(d.Cin);
  if (CinPad == 4 || d.W > 256) return 1;
  const int nchunk = CinPad / 32;
  if (nchunk < 2) return 1;
  const bool must = needs_stream(d.Cin) && (d.W & 31);          // no unsplit instance for this shape
  // Plan option fwd_csplit: 1 keeps the contraction whole where an unsplit instance exists, n >= 2 asks for n parts
  // (rounded so that a part holds at most 7 chunks); 0: the model.
  const int forced = p->opt.fwd_csplit;
  if (forced == 1 && !must) return 1;
  if (forced >= 2) {
    const int cper = std::max((nchunk + forced - 1) / forced, (nchunk + 31) / 32);
    if (cper <= 7) return (nchunk + cper - 1) / cper;
  }
  const int mode = pooled ? p4_fwd_pool_mode(p) : kOutUnpooled;
  const int nq = pooled && mode == kOutPartial ? p4_fwd_fold(p) : 1;
  long best = must ? -1 : plan_cost(p, nq > 1 ? kOutPooled : mode, 1, nq);
  int best_s = 1;
  const double part_bytes = (double)d.N * d.Cout * d.R * d.H * d.W * 4.0;
  for (int s = 2; s <= 32; s *= 2) {
    const int cper = (nchunk + s - 1) / s;
    if (cper > 7) continue;
    const int s_eff = (nchunk + cper - 1) / cper;
    if (s_eff < 2) break;
    // parts written and read once at about 4 TB/s, two small launches
    const long over = 24 + (long)(2.0 * s_eff * part_bytes / 2.0e6);
    const long c = plan_cost(p, kOutUnpooled, s_eff, 1) + over;
    if (best < 0 || c < best) { best = c; best_s = s_eff; }
    if (cper == 1) break;
  }
  return best_s;
}

// Cut the row into segments of at most 256 product columns; all segments of one launch share nwx.
// Returns the number of launches (geoms) written.
int p4_fwd_geoms(const rotconv_plan* p, int out_mode, P4Geom* out, int max_out, int csplit, int nq) {
  const rotconv_desc& d = p->d;
  P4Geom base{};
  {
    const int CinPad = cin_pad_f32(d.Cin), nchunk = CinPad == 4 ? 1 : CinPad / 32;
    base.cper = (nchunk + csplit - 1) / csplit;
    base.csplit = (nchunk + base.cper - 1) / base.cper;
  }
  base.N = d.N; base.Cin = d.Cin; base.CinPad = cin_pad_f32(d.Cin); base.H = d.H; base.W = d.W;
  base.Cout = d.Cout; base.CB = (d.Cout + 15) / 16; base.R = d.R; base.Q = p->host.Q; base.ng = p->ng;
  base.out_mode = out_mode;
  base.relu = out_mode == kOutPooled && d.activation == ROTCONV_ACT_RELU;
  int ng = 0;
  int pos = 0;
  while (pos < d.W) {
    int xorg, nwx;
    if (pos == 0) {
      xorg = 0;
      nwx = 1;
      while (nwx * 32 < d.W && nwx < 8) nwx *= 2;
    } else {
      const int need = d.W - (pos - 8);      // product columns from the pixel left of `pos` to the border
      nwx = 1;
      while (nwx * 32 < need && nwx < 8) nwx *= 2;
      // the last segment ends exactly at the right border (W % 32 == 0 here), others start 8 px early
      xorg = nwx * 32 >= need ? d.W - nwx * 32 : pos - 8;
    }
    const int chain_end = xorg + nwx * 32;
    const int hi = chain_end >= d.W ? d.W : chain_end - 8;
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
    // Rows per band: short bands cost halo rows (a band of ty rows computes ty + 2 rows of products) but give
    // more workgroups when the problem is small.  Cost of a choice = rounds of workgroups over the 256 CUs x row
    // steps per wave x how many waves share a SIMD (a workgroup whose bands reach beyond the image leaves waves idle).
    // nq > 1 (banks folded into the columns): one unit covers all banks of 16 / nq filters
    const int ublk = nq > 1 ? (d.Cout * nq + 15) / 16 : g.Q * g.CB;
    for (int ty : {1, 2, 4, 8, 16, 32, 64}) {
      const int nbg = (d.H + nwy * ty - 1) / (nwy * ty);
      const long units = (long)d.N * ublk * nbg * g.nseg * g.csplit;
      const int bands = nbg > 1 ? nwy : std::min(nwy, (d.H + ty - 1) / ty);
      const long cost = ((units + 255) / 256) * (ty + 2) * std::max(4, g.nwx * bands);
      if (best_cost < 0 || cost <= best_cost) { best_cost = cost; g.TY = ty; g.nbg = nbg; g.units = (int)units; }
    }
    g.cost = (int)std::min<long>(best_cost * g.cper, 1L << 30);
    if (nq > 1) {
      g.CB = ublk;
      g.Q = 1;
    }
    g.nq = nq;
  }
  return ng;
}

// Banks folded into a wave's 16 columns for the pooled forward: the plan pools all R = 4 Q orientations of a filter
// together, Q is 2 or 4, every bank has its four quarter turns, the channels fill whole 32-channel chunks, and the
// filter block stays LDS-resident or is streamed under rows the wave chains cover exactly (1: no folding).
int p4_fwd_fold(const rotconv_plan* p) {
  const int Q = p->host.Q;
  if ((Q != 2 && Q != 4) || p->ng != 1 || cin_pad_f32(p->d.Cin) == 4) return 1;
  // a streamed filter block: only rows that the wave chains cover exactly (the instances without load masks)
  const int W = p->d.W;
  if (needs_stream(p->d.Cin) && ((W & 31) || (W <= 256 && (W & (W - 1))))) return 1;
  for (int i = 0; i < Q * 4; ++i)
    if (p->rot_of[i] < 0) return 1;
  return Q;
}

size_t p4_fwd_pack_floats(const rotconv_plan* p) {
  return (size_t)p->host.Q * ((p->d.Cout + 15) / 16) * cin_pad_f32(p->d.Cin) * 144;
}

// How the bank kernel delivers its result for this plan's pooling.
int p4_fwd_pool_mode(const rotconv_plan* p) {
  // every bank must fall into a single pool group: all its rotations share r mod ng
  for (int q = 0; q < p->host.Q; ++q) {
    int grp = -1;
    for (int s = 0; s < 4; ++s) {
      const int r = p->rot_of[q * 4 + s];
      if (r < 0) continue;
      if (grp < 0) grp = r % p->ng;
      else if (grp != r % p->ng) return kOutUnpooled;
    }
  }
  // does a group collect more than one bank?
  return (p->host.Q > p->ng) ? kOutPartial : kOutPooled;
}

void launch_p4_pack_fwd(const rotconv_plan* p, const float* w, float* wt, hipStream_t st, int nq) {
  const int CinPad = cin_pad_f32(p->d.Cin), CB = nq > 1 ? (p->d.Cout * nq + 15) / 16 : (p->d.Cout + 15) / 16;
  const int total = (nq > 1 ? 1 : p->host.Q) * CB * CinPad * 16;
  hipLaunchKernelGGL(k_p4_pack_fwd, dim3((total + 255) / 256), dim3(256), 0, st, w, wt, p->dev.fq_src, p->dev.fq_coef,
                     p->dev.fq_coef64,
                     p->host.Q, CB, CinPad, p->d.Cin, p->d.Cout, p->d.dtype == ROTCONV_BF16 ? 1 : 0, nq);
}

bool p4_fwd_raw_weights(const rotconv_plan* p, int nq, int csplit) {
  if (p->d.dtype != ROTCONV_F32 || p->host.Q != 1 || p->B != 1 || nq > 1) return false;
  if (csplit < 2 && needs_stream(p->d.Cin)) return false;
  for (int u = 0; u < 9; ++u)
    for (int z = 0; z < kMaxNnz; ++z) {
      const int src = p->host.fq_src[u * kMaxNnz + z];
      if (z == 0 ? (src != u || p->host.fq_coef[u * kMaxNnz] != 1.0f) : src >= 0) return false;
    }
  return true;
}

void launch_p4_fwd(const rotconv_plan* p, int out_mode, const float* x, const float* wt, float* out_val,
                   uint8_t* out_idx, hipStream_t st, int nq, int csplit) {
  P4Geom gs[4];
  const int ng = p4_fwd_geoms(p, out_mode, gs, 4, csplit, nq);
  const bool stream = csplit < 2 && needs_stream(p->d.Cin);
  const int raw = p4_fwd_raw_weights(p, nq, csplit) ? 1 : 0;
  for (int i = 0; i < ng; ++i) {
    P4Geom& g = gs[i];
    g.raw_w = raw;
    const bool fastw = (p->d.W & 7) == 0 && g.inside;   // no lane reaches beyond the row: no masks, vector stores
    switch (g.nwx) {
      case 1: launch_t<1, 8>(g, fastw, stream, x, wt, p->dev.rot_of, out_val, out_idx, st); break;
      case 2: launch_t<2, 4>(g, fastw, stream, x, wt, p->dev.rot_of, out_val, out_idx, st); break;
      case 4: launch_t<4, 2>(g, fastw, stream, x, wt, p->dev.rot_of, out_val, out_idx, st); break;
      default: launch_t<8, 1>(g, fastw, stream, x, wt, p->dev.rot_of, out_val, out_idx, st); break;
    }
  }
}

void launch_p4_sum_parts(const rotconv_plan* p, const float* part, int nparts, float* y, hipStream_t st) {
  const size_t n_elem = (size_t)p->d.N * p->d.Cout * p->d.R * p->d.H * p->d.W;
  const unsigned blocks = (unsigned)std::max<size_t>(1, std::min<size_t>((n_elem / 4 + 255) / 256, 4096));
  hipLaunchKernelGGL(k_p4_sum_parts, dim3(blocks), dim3(256), 0, st, part, y, n_elem, nparts);
}

void launch_p4_sum_pool(const rotconv_plan* p, const float* part, int nparts, float* ypool, uint8_t* idx,
                        hipStream_t st) {
  const int HW = p->d.H * p->d.W;
  const size_t n_elem = (size_t)p->d.N * p->d.Cout * p->d.R * HW;
  const size_t total = (size_t)p->d.N * p->d.Cout * p->ng * HW;
  hipLaunchKernelGGL(k_p4_sum_pool, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, part, ypool, idx, n_elem,
                     nparts, p->d.N * p->d.Cout, p->d.R, p->ng, HW, p->d.activation == ROTCONV_ACT_RELU ? 1 : 0);
}

void launch_p4_combine(const rotconv_plan* p, const float* pv, const uint8_t* pi, float* ypool, uint8_t* idx,
                       hipStream_t st) {
  const int HW = p->d.H * p->d.W;
  dim3 grid((HW + 255) / 256, p->d.Cout * p->ng, p->d.N);
  hipLaunchKernelGGL(k_p4_combine, grid, dim3(256), 0, st, pv, pi, p->dev.rot_of, ypool, idx, p->d.N, p->d.Cout, HW,
                     p->host.Q, p->ng, p->d.activation == ROTCONV_ACT_RELU ? 1 : 0);
}

}  // namespace rotconv
