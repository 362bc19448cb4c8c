// Fast input-gradient kernel for 3x3, stride 1, pad 1 with bfloat16 tensors, fused with the orientation
// max-pool backward (paper Eq. 12, 13, 15) on the bf16 matrix cores, fp32 accumulation.
//
//   dX[ci,h,x] = sum_q sum_s sum_u sum_co F_q[co,ci,u] * Delta_(q,s)[co, h+1-i_s(u), x+1-j_s(u)]
//   Delta_(q,s) = G * 1[idx == orientation (q,s)],   (i_s,j_s) = R_s(u): where quarter turn s puts base tap u
//
// The fp32 kernel sums the four routed gradients at the rotated tap positions on the vector ALU before one
// contraction.  With the bf16 matrix instruction 16 times cheaper per product and vector instructions no
// cheaper, that pre-sum (and the 3x3 neighbourhood every lane had to fetch for it) would dominate, and
// its sums are not bf16 values.  Here the products are formed first, per quarter turn, on UNSHIFTED
// routed gradients, and the rotation is an index permutation on the accumulator side:
//     S_d[ci,h',x'] += sum_co F_q[co,ci,u] * Delta_(q,s)[co,h',x']      for every (s,u) with R_s(u) = d
//     dX[ci,h,x]     = sum_d S_d[ci, h+1-d_i, x+1-d_j]
// v_mfma_f32_16x16x32_bf16 with M = 16 pixels, N = 16 input channels, K = 32 filters: four quarter
// turns x nine taps = 36 products per K-step land in the nine tiles S_d (the one LDS-resident filter block
// serves all four rotations).  A lane loads one dword of G (a pixel pair of one filter) and its two idx
// bytes; routing is a compare + select per quarter turn (exact bf16 values), eight filters pack into the
// lane's K-slice of both pixel tiles.  A wave owns 16 channels x 32 pixels of a row and walks down its band
// like the forward kernel: the row of S_d feeds the output rows above, at and below through two rolling
// partial sums; column shifts are register renames plus one neighbour value per side (adjacent lane group
// via ds_bpermute, adjacent wave via LDS).  The (G, idx) rows are prefetched ND K-steps ahead through a
// register ring; a workgroup's share of the filter block [K-step][tap][k-group][16 channels][8 filters]
// is LDS-resident (at most 16 K-steps = 512 filters of one bank).
//
// Deep layers on small maps have few (channel block, band) units but a long contraction (Q * Cout
// filters): there the K-steps are split over `ksplit` workgroups per unit, each writing an fp32 partial
// dX; a second kernel adds the partials in a fixed order and rounds to bf16 (deterministic, no atomics).
// The split is also what keeps each workgroup's share of the filter block within LDS.
//
// SPARSE instances (every bank with its four quarter turns, orientations numbered r = s Q + q or r = 4 q + s): after the max-pool every (pixel,
// filter) has at most ONE non-zero quarter turn, so with the contraction index widened to (filter, quarter
// turn) the routed gradient is a 1-of-4 structured-sparse A operand and v_smfmac_f32_16x16x64_bf16 (A: 2 kept
// values of every 4 plus 2-bit positions; same cycles as the dense 16x16x32) does the four rotations' products
// in one instruction: half the matrix instructions, and routing shrinks to one validity mask per value
// plus one subtraction per destination tile.  The dense B' of destination tile d would hold F[k, ci, u_s(d)] at
// (k, s) - nine different operands; but the taps u_s(d) of the four corner destinations are the same four corner
// taps in rotated order (likewise the edges), so ONE operand per orbit, B''[(k, t)] = F[k, ci, t-th tap of the
// orbit], serves its four destinations when the position stored with the value is t = (m - s*) mod 4 for
// destination m of the orbit and winning quarter turn s*.  Operand layout of the instruction as measured on the
// chip: A lane (row, lgA) holds pairs p = 0..3 (elements 2p, 2p+1; positions in bits 4p..4p+3 of the lane's own
// index register, low / high half selected by ABID); pair p meets B lane (column, lgB = 2 (lgA % 2) + p / 2),
// elements 4 jg .. 4 jg + 3 with jg = 2 (lgA / 2) + p % 2.
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

constexpr int CHB = 9 * 4 * 16 * 8 * 2;   // bytes of one K-step (32 filters) of a 16-channel block (9216)
constexpr int CHBS = 2 * 3 * 64 * 32;     // the same in the sparse layout [half][orbit][lane][4 filters x 4 taps] (12288)
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u8x __attribute__((ext_vector_type(8)));
// destination tile of member m of an orbit (0: corners, 1: edges) = where quarter turn m puts base tap 0 / 1
__device__ __host__ constexpr int orbit_pos(int o, int m) { return tap_i(m, o) * 3 + tap_j(m, o); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{lo, hi}, bf2));
}

// ND:     K-steps the (G, idx) prefetch runs ahead (K-steps per bank are a multiple of ND).
// FASTW:  W % 8 == 0 and no wave chain reaches beyond the row: no load masks, vector stores.
// CPAD:   CoutPad > Cout: filter offsets are clamped to the last real filter (its taps are zero).
// SPLIT:  the unit's K-steps are shared by g.ksplit workgroups; the result is an fp32 partial in `part`.
// SPARSE: structured-sparse matrix instruction (see the head of the file); `wt` is in the sparse layout.
template <int NWX, int NWY, int ND, bool FASTW, bool CPAD, bool SPLIT, bool SPARSE>
__global__ __launch_bounds__(64 * NWX * NWY) void k_p4_bwd_data_bf16(const uint16_t* __restrict__ gpool,
                                                                     const uint8_t* __restrict__ idx,
                                                                     const uint16_t* __restrict__ wt,
                                                                     const int32_t* __restrict__ rot_of,
                                                                     uint16_t* __restrict__ dx,
                                                                     float* __restrict__ part, P4BwdBfGeom g) {
  constexpr int NW = NWX * NWY;
  constexpr int NT = 64 * NW;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  constexpr int KB = SPARSE ? CHBS : CHB;  // bytes of one K-step of the filter block
  char* Wl = smem_raw;                     // [kper][KB]
  const int nkc = g.CoutPad / 32;          // K-steps per bank
  const int nks = g.Q * nkc;               // K-steps per row
  float* EL = reinterpret_cast<float*>(smem_raw + g.kper * KB);  // [2][NW][3][16] left edges
  float* ER = EL + 2 * NW * 48;                                                      // right edges

  const int per_xcd = (g.units + 7) / 8;
  int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (v >= g.units) return;
  const int ksp = SPLIT ? v % g.ksplit : 0;     // fastest: the splits of a tile run side by side and share its (G, idx) lines
  if (SPLIT) v /= g.ksplit;
  const int kbeg = ksp * g.kper, kend = min(nks, kbeg + g.kper);   // this workgroup's K-steps (multiples of ND)
  const int cib = v % g.CIB; v /= g.CIB;
  const int seg = v % g.nseg; v /= g.nseg;
  const int bg = v % g.nbg;
  const int n = v / g.nbg;

  const int tid = threadIdx.x;
  const char* wsrc = reinterpret_cast<const char*>(wt) + ((size_t)cib * nks + kbeg) * KB;
  {
    const u4* src = reinterpret_cast<const u4*>(wsrc);
    u4* dst = reinterpret_cast<u4*>(Wl);
    const int n16 = (kend - kbeg) * (KB / 16);
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

  // (G, idx) loads: lane (lc, lg) reads the pixel pair x0 + 2*lc .. +1 of filter co = 32*chunk + 8*lg + j,
  // j = 0..7, in the pooled plane co*ng + (pool group of the bank).  Products of rows outside the image are
  // discarded, filters beyond Cout meet zero taps, so both only need a valid address; pixels beyond W
  // must read as zero gradient (only when W % 32 != 0).
  const int pxa = x0 + 2 * lc;
  const bool px_ok = pxa < g.W;
  const size_t img = (size_t)n * g.Cout * g.ng * HW + (px_ok ? pxa : 0);
  const uint16_t* gn = gpool + img;
  const uint8_t* in = idx + img;
  const uint32_t fstride = (uint32_t)g.ng * (uint32_t)HW;        // elements between consecutive filters
  uint32_t lgoff = (uint32_t)(8 * lg) * fstride;
  asm volatile("" : "+v"(lgoff));   // opaque: the K-step / slot part of the offset stays scalar
  const uint32_t off_last = (uint32_t)(g.Cout - 1) * fstride;
  auto row_off = [&](int t) -> uint32_t {
    const int h = min(max(y0 - 1 + t, 0), g.H - 1);
    return (uint32_t)h * (uint32_t)g.W;
  };
  // pool group of bank q: all its orientations share r mod ng
  auto group_of = [&](int q) -> int {
    int r0 = 0;
#pragma unroll
    for (int s = 3; s >= 0; --s) {
      const int r = rot_of[q * 4 + s];
      r0 = r >= 0 ? r : r0;
    }
    return r0 % g.ng;
  };
  auto load_g = [&](uint32_t base, int c, int j) -> uint32_t {   // base: row offset + pool-group plane
    uint32_t off = (uint32_t)(c * 32 + j) * fstride + lgoff;
    if (CPAD) off = min(off, off_last);
    const uint32_t v2 = *reinterpret_cast<const uint32_t*>(gn + (off + base));
    if (FASTW) return v2;
    return px_ok ? v2 : 0u;
  };
  auto load_i = [&](uint32_t base, int c, int j) -> uint32_t {
    uint32_t off = (uint32_t)(c * 32 + j) * fstride + lgoff;
    if (CPAD) off = min(off, off_last);
    return (uint32_t)*reinterpret_cast<const uint16_t*>(in + (off + base));
  };

  float accA[8], accB[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) { accA[j] = 0.f; accB[j] = 0.f; }

  // ring of ND K-step slots: slot i holds K-step (ksg + i) of the current group; refilled with the K-step
  // ND further on (of this row, or of the next row's first group) right after it has been routed
  uint32_t rg[ND][8], ri[ND][8];
  const int q_beg = kbeg / nkc, c_beg = kbeg % nkc;
  {
    const uint32_t base = row_off(0) + (uint32_t)group_of(q_beg) * (uint32_t)HW;
#pragma unroll
    for (int i = 0; i < ND; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) { rg[i][j] = load_g(base, c_beg + i, j); ri[i][j] = load_i(base, c_beg + i, j); }
    __builtin_amdgcn_s_waitcnt(0x0F70);
  }
  const char* wl_lane = Wl + lane * (SPARSE ? 32 : 16);
  // sparse routing constants.  Interleaved banks (r = s Q + q): an idx byte b belongs to bank q when b < 4 Q and
  // b % Q == q, its quarter turn is b / Q.  Bank-major (r = 4 q + s): bank b / 4, quarter turn b % 4.
  const int lq = g.bank_major ? 0 : g.Q == 4 ? 2 : g.Q == 2 ? 1 : 0;
  const uint32_t keep2 = (0xffu ^ (3u << lq)) * 0x00010001u;             // all idx bits but the quarter turn's
  const uint32_t qmul = (g.bank_major ? 4u : 1u) * 0x00010001u;         // what those bits read for bank 1

  for (int t = 0; t < nsteps; ++t) {
    const int h = y0 - 1 + t;
    const bool row_ok = h >= 0 && h < g.H;
    const uint32_t ro_cur = row_off(t), ro_nxt = row_off(t + 1);
    // S_d of this row: tile b holds pixels 2m+b.  Sparse instances: written by the row's first group (accumulator
    // input = 0); dense instances (quarter turns may be absent, so no product is known to come first): zeroed here.
    f4 S[9][2];
    const f4 zero4 = f4{0.f, 0.f, 0.f, 0.f};
    if (!SPARSE) {
#pragma unroll
      for (int d = 0; d < 9; ++d) { S[d][0] = zero4; S[d][1] = zero4; }
    }

    auto group = [&](int ksg, bool first) {
      const bool last = ksg + ND == kend;
      const int kn = last ? kbeg : ksg + ND;                // first K-step of the group being prefetched
      const int qn = kn / nkc, cn = kn % nkc;
      const uint32_t base_n = (last ? ro_nxt : ro_cur) + (uint32_t)group_of(qn) * (uint32_t)HW;
      if (SPARSE) {
        const int q = ksg / nkc;
        const uint32_t q2 = (uint32_t)q * qmul;
        const char* wc = wl_lane + (size_t)(ksg - kbeg) * CHBS;
        u8x bw[2];
        bw[0] = *reinterpret_cast<const u8x*>(wc);
#pragma unroll
        for (int i = 0; i < ND; ++i) {
          // per filter: validity mask on the pixel pair (two instructions + and), the kept value of either tile
          // (low / high half), the winning quarter turns packed as 2-bit fields (tile 0: bit 4p, tile 1: bit 16 + 4p)
          uint32_t v0[8], v1[8], sw[2] = {0u, 0u};
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const uint32_t xx = __builtin_amdgcn_perm(0u, ri[i][j], 0x0c010c00u);     // halfwords: idx of the even, odd pixel
            const uint32_t gm = rg[i][j] & match_mask2(xx & keep2, q2);
            v0[j] = gm & 0xffffu;
            v1[j] = gm >> 16;
            sw[j / 4] |= ((xx >> lq) & 0x00030003u) << (4 * (j % 4));
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int j = 0; j < 8; ++j) { rg[i][j] = load_g(base_n, cn + i, j); ri[i][j] = load_i(base_n, cn + i, j); }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            // position of the kept value for destination m of an orbit: (m - s*) mod 4, all eight fields at once
            // (4 + m - s* never borrows; the bits above a field's two land in the unused position of the zero value)
            uint32_t pos[4];
#pragma unroll
            for (int m = 0; m < 4; ++m) pos[m] = ((uint32_t)m * 0x11111111u | 0x44444444u) - sw[h];
            const bf8 a0 = __builtin_bit_cast(bf8, u4{v0[4 * h], v0[4 * h + 1], v0[4 * h + 2], v0[4 * h + 3]});
            const bf8 a1 = __builtin_bit_cast(bf8, u4{v1[4 * h], v1[4 * h + 1], v1[4 * h + 2], v1[4 * h + 3]});
#pragma unroll
            for (int o = 0; o < 3; ++o) {
              const int e = (i * 2 + h) * 3 + o;               // operand counter inside the group
              if (e + 1 < ND * 6) bw[(e + 1) & 1] = *reinterpret_cast<const u8x*>(wc + (e + 1) * 2048);
              __builtin_amdgcn_sched_barrier(0);
              const bf16x16 b = __builtin_bit_cast(bf16x16, bw[e & 1]);
              const bool init = first && i == 0 && h == 0;     // the row's first product into these tiles
              if (o < 2) {
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                  const int d = orbit_pos(o, m);
                  S[d][0] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a0, b, init ? zero4 : S[d][0], (int)pos[m], 0, 0);
                  S[d][1] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a1, b, init ? zero4 : S[d][1], (int)pos[m], 0, 1);
                }
              } else {      // centre tap: the same for every quarter turn, any position
                S[4][0] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a0, b, init ? zero4 : S[4][0], 0, 0, 0);
                S[4][1] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a1, b, init ? zero4 : S[4][1], 0, 0, 0);
              }
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        }
      } else {
        const int q = ksg / nkc;
        int rot[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) rot[s] = rot_of[q * 4 + s];
        const char* wc = wl_lane + (size_t)(ksg - kbeg) * CHB;
        u4 bw[3];
        bw[0] = *reinterpret_cast<const u4*>(wc);
        bw[1] = *reinterpret_cast<const u4*>(wc + 1024);
#pragma unroll
        for (int i = 0; i < ND; ++i) {
          // pack the eight filters' pixel pairs into the K-slices of both tiles (G and, as halfwords, idx), then
          // route per quarter turn (Eq. 12): four packed instructions per operand dword
          u4 a0[4], a1[4];
          {
            uint32_t g0[4], g1[4], x0[4], x1[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              g0[j] = __builtin_amdgcn_perm(rg[i][2 * j + 1], rg[i][2 * j], 0x05040100u);
              g1[j] = __builtin_amdgcn_perm(rg[i][2 * j + 1], rg[i][2 * j], 0x07060302u);
              x0[j] = __builtin_amdgcn_perm(ri[i][2 * j + 1], ri[i][2 * j], 0x0c040c00u);
              x1[j] = __builtin_amdgcn_perm(ri[i][2 * j + 1], ri[i][2 * j], 0x0c050c01u);
            }
#pragma unroll
            for (int s = 0; s < 4; ++s) {
              const uint32_t rs2 = (uint32_t)rot[s] * 0x00010001u;   // -1 (absent) matches no halfword
#pragma unroll
              for (int j = 0; j < 4; ++j) {
                a0[s][j] = g0[j] & match_mask2(x0[j], rs2);
                a1[s][j] = g1[j] & match_mask2(x1[j], rs2);
              }
            }
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int j = 0; j < 8; ++j) { rg[i][j] = load_g(base_n, cn + i, j); ri[i][j] = load_i(base_n, cn + i, j); }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int u = 0; u < 9; ++u) {
            const int e = i * 9 + u;
            if (e + 2 < ND * 9) bw[(e + 2) % 3] = *reinterpret_cast<const u4*>(wc + (e + 2) * 1024);
            __builtin_amdgcn_sched_barrier(0);
            const bf8 b = __builtin_bit_cast(bf8, bw[e % 3]);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
              if (rot[s] < 0) continue;                 // wave-uniform
              const int d = tap_i(s, u) * 3 + tap_j(s, u);
              S[d][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, a0[s]), b, S[d][0], 0, 0, 0);
              S[d][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, a1[s]), b, S[d][1], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    };
    // A row above / below the image (first and last band only) is multiplied like any other, from the clamped row's
    // values, and its products are then discarded; a wave whose whole band lies below the image multiplies nothing.
    if (live) {
      group(kbeg, true);
      for (int ksg = kbeg + ND; ksg < kend; ksg += ND) group(ksg, false);
    }
    if (!row_ok || !live) {
      asm volatile("" ::: "memory");       // keeps this a branch
#pragma unroll
      for (int d = 0; d < 9; ++d) { S[d][0] = zero4; S[d][1] = zero4; }
    }

    // ---- neighbour values across lane groups and waves --------------------------
    // Lane (lg, lc) holds channel lc, pixels x0 + 8*lg + j, j = 2*i + b for S[d][b][i].  Tiles with d_j = 0
    // are read one pixel to the right (need the right neighbour's first pixel), d_j = 2 one to the left.
    float nbL[3], nbR[3];  // per d_i: S_(d_i,2) at pixel (first - 1), S_(d_i,0) at pixel (last + 1)
    const int par = t & 1;
    float* el = EL + (par * NW + wave) * 48 + lc;
    float* er = ER + (par * NW + wave) * 48 + lc;
    if (lg == 0) {
#pragma unroll
      for (int di = 0; di < 3; ++di) el[di * 16] = S[di * 3][0][0];        // my first pixel of S_(di,0): for my left neighbour
    }
    if (lg == 3) {
#pragma unroll
      for (int di = 0; di < 3; ++di) er[di * 16] = S[di * 3 + 2][1][3];    // my last pixel of S_(di,2): for my right neighbour
    }
    const int addr_up = ((lane + 16) & 63) * 4, addr_dn = ((lane + 48) & 63) * 4;
#pragma unroll
    for (int di = 0; di < 3; ++di) {
      float first_px = S[di * 3][0][0], last_px = S[di * 3 + 2][1][3];
      asm volatile("" : "+v"(first_px), "+v"(last_px));    // pinned: see the forward kernel
      nbR[di] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(addr_up, __builtin_bit_cast(int, first_px)));
      nbL[di] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(addr_dn, __builtin_bit_cast(int, last_px)));
    }
    __syncthreads();
    if (NWX > 1) {
      const float* eln = EL + (par * NW + wave + 1) * 48 + lc;  // right neighbour's left edge
      const float* erp = ER + (par * NW + wave - 1) * 48 + lc;  // left neighbour's right edge
      const bool has_r = wx + 1 < NWX, has_l = wx > 0;
#pragma unroll
      for (int di = 0; di < 3; ++di) {
        const float vr = has_r ? eln[di * 16] : 0.f;
        const float vl = has_l ? erp[di * 16] : 0.f;
        nbR[di] = lg == 3 ? vr : nbR[di];
        nbL[di] = lg == 0 ? vl : nbL[di];
      }
    } else {
#pragma unroll
      for (int di = 0; di < 3; ++di) {
        nbR[di] = lg == 3 ? 0.f : nbR[di];
        nbL[di] = lg == 0 ? 0.f : nbL[di];
      }
    }

    // ---- dX[h-1] = rolling sums + this row's S_(0,.) ; rows h and h+1 keep their partial sums ----
    const int y = h - 1;                       // output row completed by this step
    const int px0 = x0 + 8 * lg;
    const int ci = cib * 16 + lc;
    const bool fin = t >= 2 && y < g.H && ci < g.Cin && px0 >= out_lo && px0 < out_hi;
    float yfin[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float tsum[3];
#pragma unroll
      for (int di = 0; di < 3; ++di) {
        // S_(di,0) at pixel j+1, S_(di,1) at pixel j, S_(di,2) at pixel j-1
        const float vr = j + 1 > 7 ? nbR[di] : S[di * 3][(j + 1) & 1][(j + 1) >> 1];
        const float vc = S[di * 3 + 1][j & 1][j >> 1];
        const float vl = j - 1 < 0 ? nbL[di] : S[di * 3 + 2][(j - 1) & 1][(j - 1) >> 1];
        tsum[di] = (vr + vc) + vl;
      }
      yfin[j] = accA[j] + tsum[0];      // product rows h-2, h-1, h are in: output row h-1 done
      accA[j] = accB[j] + tsum[1];      // output row h has product rows h-1, h
      accB[j] = tsum[2];                // output row h+1 has product row h
    }
    if (fin && SPLIT) {
      float* o = part + (((size_t)ksp * g.N + n) * g.Cin + ci) * HW + (size_t)y * g.W + px0;
      if (FASTW) {
        reinterpret_cast<f4*>(o)[0] = f4{yfin[0], yfin[1], yfin[2], yfin[3]};
        reinterpret_cast<f4*>(o)[1] = f4{yfin[4], yfin[5], yfin[6], yfin[7]};
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (px0 + j < min(g.W, out_hi)) o[j] = yfin[j];
      }
    } else if (fin) {
      uint16_t* o = dx + ((size_t)n * g.Cin + ci) * HW + (size_t)y * g.W + px0;
      if (FASTW) {
        *reinterpret_cast<u4*>(o) = u4{pack_bf16(yfin[0], yfin[1]), pack_bf16(yfin[2], yfin[3]),
                                       pack_bf16(yfin[4], yfin[5]), pack_bf16(yfin[6], yfin[7])};
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (px0 + j < min(g.W, out_hi)) o[j] = (uint16_t)(pack_bf16(yfin[j], 0.f) & 0xffffu);
      }
    }
  }
}

// dx = bf16(sum over splits, ascending, of the fp32 partials); n8 = elements / 8 (8 elements per thread).
__global__ __launch_bounds__(256) void k_p4_sum_dx_parts(const float* __restrict__ part, uint16_t* __restrict__ dx,
                                                         size_t n_elem, int ksplit) {
  const size_t n8 = n_elem / 8;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
    f4 a = reinterpret_cast<const f4*>(part)[2 * i], b = reinterpret_cast<const f4*>(part)[2 * i + 1];
    for (int k = 1; k < ksplit; ++k) {
      const f4* p = reinterpret_cast<const f4*>(part + (size_t)k * n_elem);
      a += p[2 * i];
      b += p[2 * i + 1];
    }
    reinterpret_cast<u4*>(dx)[i] = u4{pack_bf16(a[0], a[1]), pack_bf16(a[2], a[3]), pack_bf16(b[0], b[1]),
                                      pack_bf16(b[2], b[3])};
  }
  for (size_t e = n8 * 8 + (size_t)blockIdx.x * 256 + threadIdx.x; e < n_elem; e += (size_t)gridDim.x * 256) {
    float v = part[e];
    for (int k = 1; k < ksplit; ++k) v += part[(size_t)k * n_elem + e];
    dx[e] = (uint16_t)(pack_bf16(v, 0.f) & 0xffffu);
  }
}

// bf16 base bank(s) -> Q first-quadrant banks (fp32 combination rounded to bf16 once) in the LDS image layout
// of the input-gradient kernel: [16-channel block][Q][K-step of 32 filters][9 taps][4 k-groups][16 channels][8 filters].
__global__ __launch_bounds__(256) void k_p4_pack_bwd_bf16(const uint16_t* __restrict__ w, uint16_t* __restrict__ wt,
                                                          const int32_t* __restrict__ fq_src,
                                                          const double* __restrict__ fq_coef, int Q, int CIB,
                                                          int CoutPad, int Cin, int Cout) {
  // One thread per (bank, filter, channel): its nine taps read the same 18 bytes of w.
  const int total = CIB * Q * CoutPad * 16;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int c8 = e % 8;
  const int n16 = (e / 8) % 16;
  const int kg = (e / 128) % 4;
  const int chunk = (e / 512) % (CoutPad / 32);
  const int q = (e / (16 * CoutPad)) % Q;
  const int cib = e / (16 * CoutPad * Q);
  const int co = chunk * 32 + kg * 8 + c8, ci = cib * 16 + n16;
  const bool in = co < Cout && ci < Cin;
  const int slices = Cout * Cin;
  const uint16_t* src = w + (size_t)(in ? co * Cin + ci : 0) * 9;
  uint16_t* dst = wt + (size_t)(e / 512) * 4608 + e % 512;      // + u * 512
#pragma unroll
  for (int u = 0; u < 9; ++u) {
    double acc = 0.0;     // the combination in fp64, rounded to fp32 and to bf16 once each
#pragma unroll
    for (int z = 0; z < kMaxNnz; ++z) {
      const int s = fq_src[(q * 9 + u) * kMaxNnz + z];
      if (in && s >= 0)
        acc += fq_coef[(q * 9 + u) * kMaxNnz + z] * (double)bf16_to_f32(src[(size_t)(s / 9) * slices * 9 + s % 9]);
    }
    dst[u * 512] = f32_to_bf16((float)acc);
  }
}

// The same banks in the sparse layout: [16-channel block][Q][K-step][half h][orbit o][lgB][16 channels][jg][t];
// element (jg, t) of lane (lgB, channel) is tap t of orbit o (corners R_t(0), edges R_t(1), centre for every t) of
// the filter that the A lane (lgA = 2 (jg / 2) + lgB / 2) holds as pair p = 2 (lgB % 2) + jg % 2 of half h.
__global__ __launch_bounds__(256) void k_p4_pack_bwd_bf16s(const uint16_t* __restrict__ w, uint16_t* __restrict__ wt,
                                                           const int32_t* __restrict__ fq_src,
                                                           const double* __restrict__ fq_coef, int Q, int CIB,
                                                           int CoutPad, int Cin, int Cout) {
  // One thread per (bank, filter, channel): the nine taps go to three orbits x four positions (the centre four times).
  const int per_step = CHBS / 2;                      // elements of one K-step
  const int total = CIB * Q * (CoutPad / 32) * 2 * 256;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int jg = e % 4, n16 = (e / 4) % 16, lgB = (e / 64) % 4, h = (e / 256) % 2;
  const int step = e / 512;                           // (cib * Q + q) * (CoutPad / 32) + chunk
  const int chunk = step % (CoutPad / 32);
  const int q = (step / (CoutPad / 32)) % Q;
  const int cib = step / ((CoutPad / 32) * Q);
  const int lgA = 2 * (jg / 2) + lgB / 2, pr = 2 * (lgB % 2) + jg % 2;
  const int co = chunk * 32 + 8 * lgA + 4 * h + pr, ci = cib * 16 + n16;
  const bool in = co < Cout && ci < Cin;
  const int slices = Cout * Cin;
  const uint16_t* src = w + (size_t)(in ? co * Cin + ci : 0) * 9;
  float val[9];
#pragma unroll
  for (int u = 0; u < 9; ++u) {
    double acc = 0.0;     // the combination in fp64, rounded to fp32 and to bf16 once each
#pragma unroll
    for (int z = 0; z < kMaxNnz; ++z) {
      const int s = fq_src[(q * 9 + u) * kMaxNnz + z];
      if (in && s >= 0)
        acc += fq_coef[(q * 9 + u) * kMaxNnz + z] * (double)bf16_to_f32(src[(size_t)(s / 9) * slices * 9 + s % 9]);
    }
    val[u] = (float)acc;
  }
  uint16_t* dst = wt + (size_t)step * per_step + h * 3072 + lgB * 256 + n16 * 16 + jg * 4;    // + o * 1024 + t
#pragma unroll
  for (int o = 0; o < 3; ++o) {
    uint16_t t4[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) t4[t] = f32_to_bf16(val[o == 2 ? 4 : orbit_pos(o, t)]);
    *reinterpret_cast<uint2*>(dst + o * 1024) = make_uint2((uint32_t)t4[0] | ((uint32_t)t4[1] << 16), (uint32_t)t4[2] | ((uint32_t)t4[3] << 16));
  }
}

// filters padded to 32, or to a multiple of 64 (two K-steps in flight)
int cout_pad(int Cout) { return Cout <= 32 ? 32 : (Cout + 63) / 64 * 64; }
int ring_depth(int Cout) { return std::min(2, cout_pad(Cout) / 32); }
constexpr int kResidentSteps = 16;     // K-steps whose filter block fits LDS beside the edge arrays (16 * 9216 + 8192 <= 160 KB)
constexpr int kResidentStepsSparse = 12;   // 12 * 12288 + 8192 <= 160 KB

// The structured-sparse instances need every bank's four quarter turns and a regular numbering of the orientations:
// 1 = interleaved, r = s Q + q (an evenly spaced closed set), 2 = bank-major, r = 4 q + s (p4m); 0 = neither.
int sparse_order(const rotconv_plan* p) {
  const int Q = p->host.Q;
  if (Q != 1 && Q != 2 && Q != 4) return 0;
  bool inter = true, major = true;
  for (int q = 0; q < Q; ++q)
    for (int s = 0; s < 4; ++s) {
      inter = inter && p->rot_of[q * 4 + s] == s * Q + q;
      major = major && p->rot_of[q * 4 + s] == 4 * q + s;
    }
  return inter ? 1 : major ? 2 : 0;
}
bool sparse_ok(const rotconv_plan* p) { return sparse_order(p) != 0; }


template <int NWX, int NWY, int ND, bool FASTW, bool CPAD, bool SPLIT, bool SPARSE>
void launch_i(const P4BwdBfGeom& g, const uint16_t* gp, const uint8_t* idx, const uint16_t* wt, const int32_t* rot_of,
              uint16_t* dx, float* part, hipStream_t st) {
  const size_t lds = (size_t)g.kper * (SPARSE ? CHBS : CHB) + (size_t)4 * NWX * NWY * 48 * sizeof(float);
  const int grid = (g.units + 7) / 8 * 8;
  auto kern = k_p4_bwd_data_bf16<NWX, NWY, ND, FASTW, CPAD, SPLIT, SPARSE>;
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * NWX * NWY), lds, st, gp, idx, wt, rot_of, dx, part, g);
}

template <int NWX, int NWY, int ND, bool SPLIT>
void launch_t(const P4BwdBfGeom& g, bool fastw, bool cpad, bool sparse, const uint16_t* gp, const uint8_t* idx,
              const uint16_t* wt, const int32_t* rot_of, uint16_t* dx, float* part, hipStream_t st) {
  // the specialised instance: whole lanes inside the row, no padded filters; everything else takes the general one
  if (sparse) {
    if (fastw && !cpad) launch_i<NWX, NWY, ND, true, false, SPLIT, true>(g, gp, idx, wt, rot_of, dx, part, st);
    else launch_i<NWX, NWY, ND, false, true, SPLIT, true>(g, gp, idx, wt, rot_of, dx, part, st);
  } else {
    if (fastw && !cpad) launch_i<NWX, NWY, ND, true, false, SPLIT, false>(g, gp, idx, wt, rot_of, dx, part, st);
    else launch_i<NWX, NWY, ND, false, true, SPLIT, false>(g, gp, idx, wt, rot_of, dx, part, st);
  }
}

template <int NWX, int NWY>
void launch_d(int nd, const P4BwdBfGeom& g, bool fastw, bool cpad, bool sparse, const uint16_t* gp, const uint8_t* idx,
              const uint16_t* wt, const int32_t* rot_of, uint16_t* dx, float* part, hipStream_t st) {
  const bool split = g.ksplit > 1;
  if (nd == 1 && split) launch_t<NWX, NWY, 1, true>(g, fastw, cpad, sparse, gp, idx, wt, rot_of, dx, part, st);
  else if (nd == 1) launch_t<NWX, NWY, 1, false>(g, fastw, cpad, sparse, gp, idx, wt, rot_of, dx, part, st);
  else if (split) launch_t<NWX, NWY, 2, true>(g, fastw, cpad, sparse, gp, idx, wt, rot_of, dx, part, st);
  else launch_t<NWX, NWY, 2, false>(g, fastw, cpad, sparse, gp, idx, wt, rot_of, dx, part, st);
}

// Row segments and bands as in the forward kernel (rows cut into chains of at most 256 product columns
// that overlap by 8 pixels; a workgroup of 8 waves = nwx waves along x times 8 / nwx bands).
int geoms(const rotconv_plan* p, P4BwdBfGeom* out, int max_out, bool sparse) {
  const int resident = sparse ? kResidentStepsSparse : kResidentSteps;
  P4Geom fg[4];
  const int ng = p4_fwd_geoms(p, kOutPooled, fg, 4);
  if (ng < 0 || ng > max_out) return -1;
  const rotconv_desc& d = p->d;
  for (int i = 0; i < ng; ++i) {
    P4BwdBfGeom& g = out[i];
    g = P4BwdBfGeom{};
    g.N = d.N; g.Cin = d.Cin; g.CIB = (d.Cin + 15) / 16; g.H = d.H; g.W = d.W; g.Cout = d.Cout;
    g.CoutPad = cout_pad(d.Cout); g.Q = p->host.Q; g.ng = p->ng; g.bank_major = sparse_order(p) == 2;
    g.nwx = fg[i].nwx; g.nseg = fg[i].nseg; g.inside = fg[i].inside;
    for (int k = 0; k < 4; ++k) { g.seg_xorg[k] = fg[i].seg_xorg[k]; g.seg_lo[k] = fg[i].seg_lo[k]; g.seg_hi[k] = fg[i].seg_hi[k]; }
    const int nwy = 8 / g.nwx;
    long best_cost = -1;
    // bands of at least 8 rows: parallelism for small maps comes from the K split below, which costs no halo rows
    for (int ty : {8, 16, 32, 64}) {
      const int nbg = (d.H + nwy * ty - 1) / (nwy * ty);
      const long units = (long)d.N * g.CIB * nbg * g.nseg;
      const int bands = nbg > 1 ? nwy : std::min(nwy, (d.H + ty - 1) / ty);
      const long cost = ((units + 255) / 256) * (ty + 2) * std::max(4, g.nwx * bands);
      if (best_cost < 0 || cost <= best_cost) { best_cost = cost; g.TY = ty; g.nbg = nbg; g.units = (int)units; }
    }
    // Split of the K-steps over workgroups: enough workgroups to fill the chip twice, each share small enough
    // to keep its filter block LDS-resident; all segment launches of a plan use the same split (one partial
    // buffer), at most 16 parts and 256 MiB of partial sums.
    const int nd = ring_depth(d.Cout);
    const int groups = g.Q * (g.CoutPad / 32) / nd;            // prefetch groups of nd K-steps
    int want = std::max((int)((512 + g.units - 1) / g.units), (groups * nd + resident - 1) / resident);
    const double dx_bytes = 4.0 * d.N * d.Cin * d.H * d.W;
    want = std::min({want, groups, 16, std::max(1, (int)(268435456.0 / dx_bytes))});
    const int gper = (groups + want - 1) / want;               // groups per split
    g.kper = gper * nd;
    g.ksplit = (groups + gper - 1) / gper;
  }
  // one split for all launches: the coarsest
  for (int i = 1; i < ng; ++i)
    if (out[i].ksplit < out[0].ksplit) { out[0].ksplit = out[i].ksplit; out[0].kper = out[i].kper; }
  for (int i = 0; i < ng; ++i) {
    out[i].ksplit = out[0].ksplit; out[i].kper = out[0].kper;
    out[i].units *= out[i].ksplit;
  }
  return ng;
}

// The sparse instances when the orientation set allows them and their (larger) filter share fits LDS.
bool use_sparse(const rotconv_plan* p) {
  if (!sparse_ok(p)) return false;
  P4BwdBfGeom gs[4];
  return geoms(p, gs, 4, true) >= 1 && gs[0].kper <= kResidentStepsSparse;
}

}  // namespace

bool p4_bwd_data_bf16_sparse(const rotconv_plan* p) { return use_sparse(p); }

// Shapes of the forward kernel (even W, segmented rows need W % 32 == 0); every bank inside one pool group;
// after the K split a workgroup's share of the filter block must fit LDS.
bool p4_bwd_data_bf16_supported(const rotconv_plan* p) {
  if (!p4_fwd_supported(p) || !p4_bwd_data_supported(p)) return false;
  const rotconv_desc& d = p->d;
  if (d.W > 256 && (d.W & 31)) return false;
  if (use_sparse(p)) return true;
  P4BwdBfGeom gs[4];
  if (geoms(p, gs, 4, false) < 1) return false;
  return gs[0].kper <= kResidentSteps;
}

// fp32 partial sums [ksplit][N][Cin][H][W] behind the packed bank (0 when the K-steps are not split)
size_t p4_bwd_data_bf16_part_bytes(const rotconv_plan* p) {
  P4BwdBfGeom gs[4];
  if (geoms(p, gs, 4, use_sparse(p)) < 1 || gs[0].ksplit <= 1) return 0;
  return (size_t)gs[0].ksplit * p->d.N * p->d.Cin * p->d.H * p->d.W * sizeof(float);
}

size_t p4_bwd_data_bf16_pack_bytes(const rotconv_plan* p) {
  const size_t per_step = use_sparse(p) ? CHBS : CHB;
  return (size_t)((p->d.Cin + 15) / 16) * p->host.Q * (cout_pad(p->d.Cout) / 32) * per_step;
}

void launch_p4_pack_bwd_bf16(const rotconv_plan* p, const uint16_t* w, uint16_t* wt, hipStream_t st) {
  const int CIB = (p->d.Cin + 15) / 16, CoutPad = cout_pad(p->d.Cout);
  if (use_sparse(p)) {
    const int total = CIB * p->host.Q * (CoutPad / 32) * 512;
    hipLaunchKernelGGL(k_p4_pack_bwd_bf16s, dim3((total + 255) / 256), dim3(256), 0, st, w, wt, p->dev.fq_src,
                       p->dev.fq_coef64, p->host.Q, CIB, CoutPad, p->d.Cin, p->d.Cout);
    return;
  }
  const int total = CIB * p->host.Q * CoutPad * 16;
  hipLaunchKernelGGL(k_p4_pack_bwd_bf16, dim3((total + 255) / 256), dim3(256), 0, st, w, wt, p->dev.fq_src,
                     p->dev.fq_coef64, p->host.Q, CIB, CoutPad, p->d.Cin, p->d.Cout);
}

// part: scratch of p4_bwd_data_bf16_part_bytes() bytes (unused when that is 0)
void launch_p4_bwd_data_bf16(const rotconv_plan* p, const uint16_t* gpool, const uint8_t* idx, const uint16_t* wt,
                             uint16_t* dx, float* part, hipStream_t st) {
  P4BwdBfGeom gs[4];
  const bool sparse = use_sparse(p);
  const int ng = geoms(p, gs, 4, sparse);
  const int nd = ring_depth(p->d.Cout);
  for (int i = 0; i < ng; ++i) {
    const P4BwdBfGeom& g = gs[i];
    const bool fastw = (p->d.W & 7) == 0 && g.inside;
    const bool cpad = g.CoutPad != p->d.Cout;
    switch (g.nwx) {
      case 1: launch_d<1, 8>(nd, g, fastw, cpad, sparse, gpool, idx, wt, p->dev.rot_of, dx, part, st); break;
      case 2: launch_d<2, 4>(nd, g, fastw, cpad, sparse, gpool, idx, wt, p->dev.rot_of, dx, part, st); break;
      case 4: launch_d<4, 2>(nd, g, fastw, cpad, sparse, gpool, idx, wt, p->dev.rot_of, dx, part, st); break;
      default: launch_d<8, 1>(nd, g, fastw, cpad, sparse, gpool, idx, wt, p->dev.rot_of, dx, part, st); break;
    }
  }
  if (ng > 0 && gs[0].ksplit > 1) {
    const size_t n_elem = (size_t)p->d.N * p->d.Cin * p->d.H * p->d.W;
    const unsigned blocks = (unsigned)std::max<size_t>(1, std::min<size_t>((n_elem / 8 + 255) / 256, 1u << 16));
    hipLaunchKernelGGL(k_p4_sum_dx_parts, dim3(blocks), dim3(256), 0, st, part, dx, n_elem, gs[0].ksplit);
  }
}

}  // namespace rotconv
