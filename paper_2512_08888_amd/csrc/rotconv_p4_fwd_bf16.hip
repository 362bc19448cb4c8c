// Fast forward kernel for 3x3, stride 1, pad 1 with bfloat16 tensors: shared-product rotation
// convolution (paper Eq. 8) on the bf16 matrix cores, fp32 accumulation.
//
// Same decomposition as the fp32 kernel: per first-quadrant bank the nine per-tap channel
// contractions P_u[co,h,x] = sum_ci F[co,ci,u] X[ci,h,x] are formed once, here with
// v_mfma_f32_16x16x32_bf16 (M = 16 pixels, N = 16 filters, K = 32 input channels), and placed at the
// four quarter-turn positions in registers; max / arg-max over the bank's rotations are taken on the
// fp32 sums and the winner is rounded to bf16 once.  A wave owns 16 filters x 32 consecutive pixels
// of one row and walks down its band of rows.
//
// What differs from the fp32 kernel is the operand feed.  A lane loads one dword = the pixel pair
// (2m, 2m+1) of one channel; eight channels give, after eight byte permutes, the lane's K-slice of
// both pixel tiles.  With 32 channels per matrix instruction the contraction of a 32-channel chunk
// is only 18 instructions of 16 clocks, far shorter than the memory latency, so the input rows are
// prefetched ND = 2 chunks (64 channels) ahead through a ring of register slots, across row ends.
// The filter block [chunk][tap][k-group][filter][8 channels] sits in LDS (one 16-byte read per lane
// and tap, conflict free); blocks deeper than 480 channels are streamed in stages of ND chunks.
// With the contraction this cheap the kernel is bound by the placement adds on the vector ALU.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "rotconv_bf16.h"
#include "rotconv_kernels.h"
#include "rotconv_p4.h"
#include "rotconv_p4_taps.h"

namespace rotconv {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));

constexpr int CHB = 9 * 4 * 16 * 8 * 2;   // bytes of one 32-channel chunk of a 16-filter block (9216)

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{lo, hi}, bf2));
}

// ND:       chunks of 32 channels the input prefetch runs ahead (CinPad is a multiple of 32 * ND).
// UNPOOLED: write every orientation (rotconv_fwd); else max + arg-max over the bank's rotations.
// FASTW:    W % 8 == 0 and no wave chain reaches beyond the row: no load masks, vector stores.
// STREAM:   the filter block does not fit LDS: stream it in stages of ND chunks.
// CPAD:     CinPad > Cin: channel offsets are clamped to the last real channel (its taps are zero).
// NQ:       banks folded into the 16 filter columns of a wave (1, 2 or 4).  NQ > 1 is for a pool group that spans
//           all NQ banks of the plan (R = 4 NQ orientations pooled together): column n holds bank n / (16/NQ),
//           filter n % (16/NQ), every lane places and maximises its own bank's four rotations, and the maximum
//           across the banks is a rotate-and-compare inside the 16-lane row (DPP) - the per-bank candidates
//           never go through memory.  Pooled output only; every bank has all four quarter turns.
template <int NWX, int NWY, int ND, bool UNPOOLED, bool FASTW, bool STREAM, bool CPAD, int NQ>
__global__ __launch_bounds__(64 * NWX * NWY) void k_p4_fwd_bf16(const uint16_t* __restrict__ x,
                                                                const uint16_t* __restrict__ wt,
                                                                const int32_t* __restrict__ rot_of,
                                                                void* __restrict__ out_val,
                                                                uint8_t* __restrict__ out_idx, P4Geom g) {
  constexpr int NW = NWX * NWY;
  constexpr int NT = 64 * NW;
  constexpr int STB = ND * CHB;            // bytes of one streaming stage
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  char* Wl = smem_raw;                     // resident: [nchunk][CHB]; streamed: [2][STB]
  const int nchunk = g.CinPad / 32;
  float* EL = reinterpret_cast<float*>(smem_raw + (STREAM ? 2 * STB : nchunk * CHB));  // [2][NW][8][16]
  float* ER = EL + 2 * NW * 128;

  // XCD-aware unit decode: consecutive units (same image rows, different filter blocks / banks) go to
  // the same XCD so they share its L2 copy of the input.
  const int per_xcd = (g.units + 7) / 8;
  int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (v >= g.units) return;
  const int cb = v % g.CB; v /= g.CB;
  const int q = v % g.Q; v /= g.Q;
  const int seg = v % g.nseg; v /= g.nseg;
  const int bg = v % g.nbg;
  const int n = v / g.nbg;

  const int tid = threadIdx.x;
  const char* wsrc = reinterpret_cast<const char*>(wt) + (size_t)(q * g.CB + cb) * nchunk * CHB;
  constexpr int WPT = (STB / 16 + NT - 1) / NT;   // 16-byte units per thread and stage when streaming
  u4 wreg[STREAM ? WPT : 1];
  auto wload = [&](int stage) {
#pragma unroll
    for (int k = 0; k < WPT; ++k) {
      const int e = tid + k * NT;
      if (e < STB / 16) wreg[k] = reinterpret_cast<const u4*>(wsrc + (size_t)stage * STB)[e];
    }
  };
  auto wstore = [&](int buf) {
#pragma unroll
    for (int k = 0; k < WPT; ++k) {
      const int e = tid + k * NT;
      if (e < STB / 16) reinterpret_cast<u4*>(Wl + buf * STB)[e] = wreg[k];
    }
  };
  if (STREAM) {
    wload(0);
    wstore(0);
  } else {
    const u4* src = reinterpret_cast<const u4*>(wsrc);
    u4* dst = reinterpret_cast<u4*>(Wl);
    const int n16 = nchunk * (CHB / 16);
    for (int i = tid; i < n16; i += NT) dst[i] = src[i];
  }
  __syncthreads();

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

  // A-operand loads: lane (lc, lg) reads the dword X[ci = 32*chunk + 8*lg + j][h][x0 + 2*lc .. +1],
  // j = 0..7.  Products of rows outside the image are discarded, channels beyond Cin meet zero taps, so both
  // only need a valid address; pixels beyond W must read as zero (only when W % 32 != 0).
  const int pxa = x0 + 2 * lc;
  const bool px_ok = pxa < g.W;
  // address = wave-uniform part (image, row, chunk and slot channel: scalar registers) + one per-lane byte offset
  // that never changes (pixel pair, k-group's channels), so a load costs no vector arithmetic
  const uint16_t* xn = x + (size_t)n * g.Cin * HW;
  const uint32_t lgoff = (uint32_t)(8 * lg) * (uint32_t)HW;
  const uint32_t lane_off = 2u * (lgoff + (uint32_t)(px_ok ? pxa : 0));
  const uint32_t off_last = (uint32_t)(g.Cin - 1) * (uint32_t)HW;
  auto row_ptr = [&](int t) -> const uint16_t* {
    const int h = min(max(y0 - 1 + t, 0), g.H - 1);
    return xn + (size_t)h * g.W;
  };
  const size_t plane_bytes = (size_t)HW * 2;
  // the eight channels of chunk c that this lane's k-group feeds, into dst[0..7]
  auto load_chunk = [&](const uint16_t* rp, int c, uint32_t* dst) {
    if (CPAD) {     // channels beyond Cin read the last one (their taps are zero)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint32_t off = min((uint32_t)(c * 32 + j) * (uint32_t)HW + lgoff, off_last) + (uint32_t)(px_ok ? pxa : 0);
        dst[j] = *reinterpret_cast<const uint32_t*>(rp + off);
      }
    } else {
      const char* base = reinterpret_cast<const char*>(rp) + (size_t)(c * 32) * plane_bytes;   // scalar
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        dst[j] = *reinterpret_cast<const uint32_t*>(base + lane_off);
        base += plane_bytes;
      }
    }
    if (!FASTW) {
#pragma unroll
      for (int j = 0; j < 8; ++j) dst[j] = px_ok ? dst[j] : 0u;
    }
  };

  float accA[4][8], accB[4][8];
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int j = 0; j < 8; ++j) { accA[s][j] = 0.f; accB[s][j] = 0.f; }

  // ring of ND chunk slots: slot i holds chunk (cc + i) of the current group; it is refilled with the
  // chunk ND further on (of this row, or of the next row's first group) right after it has been packed
  uint32_t ring[ND][8];
  {
    const uint16_t* rp = row_ptr(0);
#pragma unroll
    for (int i = 0; i < ND; ++i) load_chunk(rp, i, ring[i]);
    __builtin_amdgcn_s_waitcnt(0x0F70);
  }
  const char* wl_lane = Wl + lane * 16;
  int seq = 0;                           // groups done (streaming: LDS buffer parity)

  for (int t = 0; t < nsteps; ++t) {
    const int h = y0 - 1 + t;
    const bool row_ok = h >= 0 && h < g.H;
    const uint16_t* rp_cur = row_ptr(t);
    const uint16_t* rp_nxt = row_ptr(t + 1);
    f4 P[9][2];

    // One group of ND chunks.  Per chunk: pack the slot into the two tiles' A operands, refill the
    // slot, then 9 taps x 2 tiles of matrix instructions with the B operand read from LDS two taps
    // ahead.  Scheduling fences keep loads and LDS reads where they are issued.
    auto group = [&](int cc, bool first) {
      const bool last = cc + ND == nchunk;
      const uint16_t* rp = last ? rp_nxt : rp_cur;
      const int cn = last ? 0 : cc + ND;
      if (STREAM) wload(last ? 0 : cc / ND + 1);
      const char* wc = STREAM ? wl_lane + (seq & 1) * STB : wl_lane + (size_t)cc * CHB;
      u4 bw[3];
      bw[0] = *reinterpret_cast<const u4*>(wc);
      bw[1] = *reinterpret_cast<const u4*>(wc + 1024);
#pragma unroll
      for (int i = 0; i < ND; ++i) {
        u4 a0, a1;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          a0[j] = __builtin_amdgcn_perm(ring[i][2 * j + 1], ring[i][2 * j], 0x05040100u);
          a1[j] = __builtin_amdgcn_perm(ring[i][2 * j + 1], ring[i][2 * j], 0x07060302u);
        }
        __builtin_amdgcn_sched_barrier(0);
        load_chunk(rp, cn + i, ring[i]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 9; ++u) {
          const int e = i * 9 + u;               // tap counter inside the group
          if (e + 2 < ND * 9) bw[(e + 2) % 3] = *reinterpret_cast<const u4*>(wc + (e + 2) * 1024);
          __builtin_amdgcn_sched_barrier(0);
          const f4 zero = f4{0.f, 0.f, 0.f, 0.f};
          const bf8 b = __builtin_bit_cast(bf8, bw[e % 3]);
          P[u][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, a0), b,
                                                            first && i == 0 ? zero : P[u][0], 0, 0, 0);
          P[u][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, a1), b,
                                                            first && i == 0 ? zero : P[u][1], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
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
      group(0, true);
      for (int cc = ND; cc < nchunk; cc += ND) group(cc, false);
    } else if (STREAM) {
      for (int cc = 0; cc < nchunk; cc += ND) {
        wload(cc + ND == nchunk ? 0 : cc / ND + 1);
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
      // sources pinned in VGPRs of their own: an accumulator element handed straight to the
      // cross-lane read selected the wrong element
      float first_px = P[u][0][0], last_px = P[u][1][3];
      asm volatile("" : "+v"(first_px), "+v"(last_px));
      nbR[u] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(addr_up, __builtin_bit_cast(int, first_px)));
      nbL[u] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(addr_dn, __builtin_bit_cast(int, last_px)));
    }
    __syncthreads();
    if (NWX > 1) {
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
    bool none = true;
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
    auto store8_bf16 = [&](uint16_t* o, const float* v8) {
      if (FASTW) {
        *reinterpret_cast<u4*>(o) = u4{pack_bf16(v8[0], v8[1]), pack_bf16(v8[2], v8[3]), pack_bf16(v8[4], v8[5]),
                                       pack_bf16(v8[6], v8[7])};
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (px0 + j < min(g.W, out_hi)) o[j] = (uint16_t)(pack_bf16(v8[j], 0.f) & 0xffffu);
      }
    };
    if (UNPOOLED) {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        float yfin[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) place(s, j, yfin[j]);
        if (fin && rot[s] >= 0)
          store8_bf16(static_cast<uint16_t*>(out_val) + (((size_t)n * g.Cout + co) * g.R + rot[s]) * HW +
                          (size_t)y * g.W + px0, yfin);
      }
    } else {
      if (NQ == 1) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
          if (rot[s] >= 0) { grp_r = rot[s]; none = false; }
      } else {
        none = false;       // all rotations present, one pool group (channel = co)
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
          auto other = [&](int ctrl_v, int ctrl_i) {
            const float ov = __builtin_bit_cast(float, ctrl_v);
            const bool take = ov > bv || (ov == bv && ctrl_i < bi);     // ties: the smallest orientation index
            bv = take ? ov : bv;
            bi = take ? ctrl_i : bi;
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
    if (!UNPOOLED && fin && !none) {
      if (g.out_mode == kOutPooled) {
        // every rotation of this bank lies in pool group (r mod ng); pooled channel = co*ng + group
        const size_t chan = (size_t)n * g.Cout * g.ng + (size_t)co * g.ng + (grp_r % g.ng);
        const size_t off = chan * HW + (size_t)y * g.W + px0;
        store8_bf16(static_cast<uint16_t*>(out_val) + off, best);
        if (FASTW) {
          *reinterpret_cast<uint2*>(out_idx + off) = make_uint2(pk[0], pk[1]);
        } else {
#pragma unroll
          for (int j = 0; j < 8; ++j)
            if (px0 + j < min(g.W, out_hi)) out_idx[off + j] = (uint8_t)(pk[j >> 2] >> (8 * (j & 3)));
        }
      } else {  // kOutPartial: per-bank fp32 candidates [Q][N][Cout][H][W] (the max across banks is taken on fp32)
        const size_t chan = ((size_t)q * g.N + n) * g.Cout + co;
        const size_t off = chan * HW + (size_t)y * g.W + px0;
        float* ov = static_cast<float*>(out_val);
        if (FASTW) {
          f4* o = reinterpret_cast<f4*>(ov + off);
          o[0] = f4{best[0], best[1], best[2], best[3]};
          o[1] = f4{best[4], best[5], best[6], best[7]};
          *reinterpret_cast<uint2*>(out_idx + off) = make_uint2(pk[0], pk[1]);
        } else {
#pragma unroll
          for (int j = 0; j < 8; ++j)
            if (px0 + j < min(g.W, out_hi)) {
              ov[off + j] = best[j];
              out_idx[off + j] = (uint8_t)(pk[j >> 2] >> (8 * (j & 3)));
            }
        }
      }
    }
  }
}

// Max over the per-bank fp32 candidates of a pool group that spans several banks, rounded to bf16.
// Candidates [Q][N][Cout][HW]; group g of filter co collects banks q with (r mod ng) == g.
__global__ __launch_bounds__(256) void k_p4_combine_bf16(const float* __restrict__ pv, const uint8_t* __restrict__ pi,
                                                         const int32_t* __restrict__ rot_of,
                                                         uint16_t* __restrict__ ypool, uint8_t* __restrict__ idx, int N,
                                                         int Cout, int HW, int Q, int ng, int relu) {
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
  ypool[o] = dead ? (uint16_t)0 : f32_to_bf16(best);
  idx[o] = dead ? (uint8_t)255 : (uint8_t)bi;
}

// bf16 base bank(s) -> Q first-quadrant banks (Sec. III-D / Eq. 17 combination in fp64, rounded to fp32 and
// to bf16 once each) in the LDS image layout [Q][CB][chunk][9 taps][4 k-groups][16 filters][8 channels]; zero for
// padded filters / channels.
// nq > 1: the banks are folded into the 16 columns (column n = bank n / (16/nq), filter n % (16/nq)): [CB'][chunk]...
// One thread per (filter, channel): it reads the 9 NB taps of its base filter(s) once and forms all Q banks with
// wave-uniform fp64 coefficients (dense [Q][9][NS] matrices, NS = 9 source taps per base bank).
template <int NS>
__global__ __launch_bounds__(256) void k_p4_pack_fwd_bf16(const uint16_t* __restrict__ w, uint16_t* __restrict__ wt,
                                                          const double* __restrict__ dense, int Q, int CB, int CinPad,
                                                          int Cin, int Cout, int nq) {
  const int fpb = nq > 1 ? 16 / nq : 16;                 // filters of a block that are distinct filters
  const int total = CB * CinPad * fpb;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int c8 = e % 8;
  const int fs = (e / 8) % fpb;
  const int kg = (e / (8 * fpb)) % 4;
  const int chunk = (e / (32 * fpb)) % (CinPad / 32);
  const int cb = e / (fpb * CinPad);
  const int co = cb * fpb + fs, ci = chunk * 32 + kg * 8 + c8;
  const bool in = co < Cout && ci < Cin;
  const size_t slices = (size_t)Cout * Cin;
  const uint16_t* src = w + (size_t)(in ? co * Cin + ci : 0) * 9;
  double wv[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) wv[s] = in ? (double)bf16_to_f32(src[(size_t)(s / 9) * slices * 9 + s % 9]) : 0.0;
  for (int q = 0; q < Q; ++q) {
    const int f16 = nq > 1 ? q * fpb + fs : fs;
    const int blk = nq > 1 ? cb : q * CB + cb;
    uint16_t* dst = wt + ((size_t)blk * (CinPad / 32) + chunk) * 4608 + (kg * 16 + f16) * 8 + c8;      // + u * 512
    const double* dq = dense + (size_t)q * 9 * NS;
#pragma unroll
    for (int u = 0; u < 9; ++u) {
      double acc = 0.0;     // the combination in fp64, rounded to fp32 and to bf16 once each
#pragma unroll
      for (int s = 0; s < NS; ++s) acc += dq[u * NS + s] * wv[s];
      dst[u * 512] = f32_to_bf16((float)acc);
    }
  }
}

// the ring holds two chunks (a deeper one spills registers): channels padded to a multiple of 64 beyond 32
int cin_pad(int Cin) { return Cin <= 32 ? 32 : (Cin + 63) / 64 * 64; }
int ring_depth(int Cin) { return std::min(2, cin_pad(Cin) / 32); }
// Is the filter block of 16 filters too large to stay in LDS next to the edge arrays?
bool needs_stream(int Cin) { return (size_t)(cin_pad(Cin) / 32) * CHB + 16384 > 160 * 1024; }

template <int NWX, int NWY, int ND, bool UNPOOLED, bool FASTW, bool STREAM, bool CPAD, int NQ = 1>
void launch_i(const P4Geom& g, const uint16_t* x, const uint16_t* wt, const int32_t* rot_of, void* ov, uint8_t* oi,
              hipStream_t st) {
  const size_t wbytes = STREAM ? (size_t)2 * ND * CHB : (size_t)(g.CinPad / 32) * CHB;
  const size_t lds = wbytes + (size_t)4 * NWX * NWY * 128 * sizeof(float);
  const int grid = (g.units + 7) / 8 * 8;
  auto kern = k_p4_fwd_bf16<NWX, NWY, ND, UNPOOLED, FASTW, STREAM, CPAD, NQ>;
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * NWX * NWY), lds, st, x, wt, rot_of, ov, oi, g);
}

template <int NWX, int NWY, int ND>
void launch_t(const P4Geom& g, bool fastw, bool stream, bool cpad, const uint16_t* x, const uint16_t* wt,
              const int32_t* rot_of, void* ov, uint8_t* oi, hipStream_t st) {
  const bool unp = g.out_mode == kOutUnpooled;
  if (g.nq > 1) {       // banks folded into the columns: resident filter block, pooled output
    if (g.nq == 4) {
      if (fastw && !cpad) launch_i<NWX, NWY, ND, false, true, false, false, 4>(g, x, wt, rot_of, ov, oi, st);
      else launch_i<NWX, NWY, ND, false, false, false, true, 4>(g, x, wt, rot_of, ov, oi, st);
    } else {
      if (fastw && !cpad) launch_i<NWX, NWY, ND, false, true, false, false, 2>(g, x, wt, rot_of, ov, oi, st);
      else launch_i<NWX, NWY, ND, false, false, false, true, 2>(g, x, wt, rot_of, ov, oi, st);
    }
    return;
  }
  // the specialised instances: pooled output, whole lanes inside the row; everything else takes the
  // general instance (masks, clamped channels)
  if (unp && stream) launch_i<NWX, NWY, ND, true, false, true, true>(g, x, wt, rot_of, ov, oi, st);
  else if (unp) launch_i<NWX, NWY, ND, true, false, false, true>(g, x, wt, rot_of, ov, oi, st);
  else if (stream && fastw) launch_i<NWX, NWY, ND, false, true, true, false>(g, x, wt, rot_of, ov, oi, st);
  else if (stream) launch_i<NWX, NWY, ND, false, false, true, false>(g, x, wt, rot_of, ov, oi, st);
  else if (fastw && !cpad) launch_i<NWX, NWY, ND, false, true, false, false>(g, x, wt, rot_of, ov, oi, st);
  else launch_i<NWX, NWY, ND, false, false, false, true>(g, x, wt, rot_of, ov, oi, st);
}

template <int NWX, int NWY>
void launch_d(int nd, const P4Geom& g, bool fastw, bool stream, bool cpad, const uint16_t* x, const uint16_t* wt,
              const int32_t* rot_of, void* ov, uint8_t* oi, hipStream_t st) {
  switch (nd) {
    case 1: launch_t<NWX, NWY, 1>(g, fastw, stream, cpad, x, wt, rot_of, ov, oi, st); break;
    default: launch_t<NWX, NWY, 2>(g, fastw, stream, cpad, x, wt, rot_of, ov, oi, st); break;
  }
}

}  // namespace

// Banks folded into a wave's 16 columns: the plan pools all R = 4 Q orientations of a filter together, Q is 2 or
// 4, every bank has its four quarter turns, and the filter block stays LDS-resident.  Then the pooled forward
// needs no per-bank candidates.
int p4_fwd_bf16_fold(const rotconv_plan* p) {
  const int Q = p->host.Q;
  if ((Q != 2 && Q != 4) || p->ng != 1 || needs_stream(p->d.Cin)) return 1;
  for (int i = 0; i < Q * 4; ++i)
    if (p->rot_of[i] < 0) return 1;
  return Q;
}

// The bf16 kernel covers the fp32 kernel's shapes; the streamed variant (Cin > 480) is built for whole
// lanes inside the row and unpadded channel counts.
bool p4_fwd_bf16_supported(const rotconv_plan* p) {
  if (!p4_fwd_supported(p)) return false;
  const rotconv_desc& d = p->d;
  if (needs_stream(d.Cin) && ((d.W & 31) || cin_pad(d.Cin) != d.Cin)) return false;
  return true;
}

size_t p4_fwd_bf16_pack_bytes(const rotconv_plan* p) {
  return (size_t)p->host.Q * ((p->d.Cout + 15) / 16) * cin_pad(p->d.Cin) * 144 * sizeof(uint16_t);
}

// nq: 1 = one bank per wave ([Q][CB] blocks); p4_fwd_bf16_fold(p) = banks folded into the columns ([CB'] blocks)
void launch_p4_pack_fwd_bf16(const rotconv_plan* p, int nq, const uint16_t* w, uint16_t* wt, hipStream_t st) {
  const int CinPad = cin_pad(p->d.Cin), CB = nq > 1 ? (p->d.Cout * nq + 15) / 16 : (p->d.Cout + 15) / 16;
  const int total = CB * CinPad * (nq > 1 ? 16 / nq : 16);
  if (p->B == 1)
    hipLaunchKernelGGL(k_p4_pack_fwd_bf16<9>, dim3((total + 255) / 256), dim3(256), 0, st, w, wt, p->dev.fq_dense64,
                       p->host.Q, CB, CinPad, p->d.Cin, p->d.Cout, nq);
  else
    hipLaunchKernelGGL(k_p4_pack_fwd_bf16<18>, dim3((total + 255) / 256), dim3(256), 0, st, w, wt, p->dev.fq_dense64,
                       p->host.Q, CB, CinPad, p->d.Cin, p->d.Cout, nq);
}

// out_val: bf16 [N][C'][H][W] (kOutPooled), bf16 [N][Cout*R][H][W] (kOutUnpooled) or fp32 per-bank
// candidates (kOutPartial).
// nq > 1 (only with kOutPooled): wt holds the folded blocks and the kernel pools across the banks itself.
void launch_p4_fwd_bf16(const rotconv_plan* p, int out_mode, int nq, const uint16_t* x, const uint16_t* wt, void* out_val,
                        uint8_t* out_idx, hipStream_t st) {
  P4Geom gs[4];
  const int ng = p4_fwd_geoms(p, out_mode, gs, 4);
  const bool stream = needs_stream(p->d.Cin);
  const int nd = ring_depth(p->d.Cin);
  for (int i = 0; i < ng; ++i) {
    P4Geom& g = gs[i];
    g.CinPad = cin_pad(p->d.Cin);
    g.nq = nq;
    if (nq > 1) {         // one unit covers all banks of 16 / nq filters
      const int CBf = (p->d.Cout * nq + 15) / 16;
      g.units = g.units / (g.Q * g.CB) * CBf;
      g.CB = CBf;
      g.Q = 1;
    }
    const bool fastw = (p->d.W & 7) == 0 && g.inside;
    const bool cpad = g.CinPad != p->d.Cin;
    switch (g.nwx) {
      case 1: launch_d<1, 8>(nd, g, fastw, stream, cpad, x, wt, p->dev.rot_of, out_val, out_idx, st); break;
      case 2: launch_d<2, 4>(nd, g, fastw, stream, cpad, x, wt, p->dev.rot_of, out_val, out_idx, st); break;
      case 4: launch_d<4, 2>(nd, g, fastw, stream, cpad, x, wt, p->dev.rot_of, out_val, out_idx, st); break;
      default: launch_d<8, 1>(nd, g, fastw, stream, cpad, x, wt, p->dev.rot_of, out_val, out_idx, st); break;
    }
  }
}

void launch_p4_combine_bf16(const rotconv_plan* p, const float* pv, const uint8_t* pi, uint16_t* ypool, uint8_t* idx,
                            hipStream_t st) {
  const int HW = p->d.H * p->d.W;
  dim3 grid((HW + 255) / 256, p->d.Cout * p->ng, p->d.N);
  hipLaunchKernelGGL(k_p4_combine_bf16, grid, dim3(256), 0, st, pv, pi, p->dev.rot_of, ypool, idx, p->d.N, p->d.Cout,
                     HW, p->host.Q, p->ng, p->d.activation == ROTCONV_ACT_RELU ? 1 : 0);
}

}  // namespace rotconv
