// Declarations of the fast (MFMA, 3x3 / stride 1 / pad 1) kernel family.
#pragma once

#include <hip/hip_runtime.h>

#include "rotconv_internal.h"

namespace rotconv {

enum { kOutPooled = 0, kOutPartial = 1, kOutUnpooled = 2 };

struct P4Geom {
  int N, Cin, CinPad, H, W, Cout, CB, R, Q, ng;
  int TY;        // output rows per wave band
  int nbg;       // band groups per image (a workgroup takes NWY consecutive bands)
  int units;     // workgroups with work
  int nwx;       // waves along x
  int out_mode;  // kOut*
  int nseg;      // row segments handled by this launch (1 unless W > 256)
  int inside;    // 1 if no segment's wave chain reaches beyond the row
  int relu;      // pooled output: clamp at 0, idx 255 where the pooled value is not positive
  int nq;        // banks folded into a wave's 16 filter columns (0 / 1: none)
  int csplit;    // parts the channel contraction is split into (1: none); a part is an unpooled fp32 map
  int cper;      // 32-channel chunks per part (all of them without a split)
  int cost;      // modelled cost of the launch (host side only)
  int raw_w;     // the weight argument is the caller's w[Cout][Cin][9] itself (see p4_fwd_raw_weights)
  int seg_xorg[4];  // first product column of a segment's wave chain
  int seg_lo[4], seg_hi[4];  // output pixels [lo, hi) the segment stores (multiples of 8, or W)
};

// forward
bool p4_fwd_supported(const rotconv_plan* p);
int p4_fwd_geoms(const rotconv_plan* p, int out_mode, P4Geom* out, int max_out, int csplit = 1, int nq = 1);
// parts the forward splits its channel contraction into for this plan (1: none); with a split the kernel runs in
// the unpooled mode into `csplit` parts of N * Cout * R * H * W floats, added by one of the two kernels below
int p4_fwd_csplit(const rotconv_plan* p, bool pooled);
void launch_p4_sum_parts(const rotconv_plan* p, const float* part, int nparts, float* y, hipStream_t st);
void launch_p4_sum_pool(const rotconv_plan* p, const float* part, int nparts, float* ypool, uint8_t* idx,
                        hipStream_t st);   // applies the plan's fused activation
size_t p4_fwd_pack_floats(const rotconv_plan* p);
int p4_fwd_pool_mode(const rotconv_plan* p);
int p4_fwd_fold(const rotconv_plan* p);   // banks a wave can fold into its columns for the pooled forward (1: none)
// nq = 1: one bank per wave; nq = p4_fwd_fold(p) > 1 (with kOutPooled): folded blocks, pooled across banks in-kernel
void launch_p4_pack_fwd(const rotconv_plan* p, const float* w, float* wt, hipStream_t st, int nq = 1);
// A plan whose one bank is its base bank (exact quarter turns, or a single orientation) and whose filter block stays in
// LDS: the forward kernel re-lays its block out of the caller's weights itself, launch_p4_fwd takes w in place of the
// packed bank and launch_p4_pack_fwd is not called (one small dependent launch less per call).
bool p4_fwd_raw_weights(const rotconv_plan* p, int nq = 1, int csplit = 1);
void launch_p4_fwd(const rotconv_plan* p, int out_mode, const float* x, const float* wt, float* out_val,
                   uint8_t* out_idx, hipStream_t st, int nq = 1, int csplit = 1);
void launch_p4_combine(const rotconv_plan* p, const float* pv, const uint8_t* pi, float* ypool, uint8_t* idx,
                       hipStream_t st);   // applies the plan's fused activation

// pooled forward on base products (pool group spanning several banks): one conv-equivalent on the matrix cores
int p4_fwd_base_classify(const rotconv_plan* p, std::vector<float>* coef);   // bank classes (-1: none) and coefficients
bool p4_fwd_base_supported(const rotconv_plan* p);
size_t p4_fwd_base_pack_floats(const rotconv_plan* p);
void launch_p4_pack_base(const rotconv_plan* p, const float* w, float* wt, hipStream_t st);
void launch_p4_fwd_base(const rotconv_plan* p, const float* x, const float* wt, float* ypool, uint8_t* idx,
                        hipStream_t st);

// forward on bfloat16 tensors (bf16 matrix cores, fp32 accumulation); out_val is bf16 for the pooled and
// unpooled modes and fp32 for the per-bank candidates
bool p4_fwd_bf16_supported(const rotconv_plan* p);
size_t p4_fwd_bf16_pack_bytes(const rotconv_plan* p);
int p4_fwd_bf16_fold(const rotconv_plan* p);   // banks a wave can fold into its columns for the pooled forward (1: none)
void launch_p4_pack_fwd_bf16(const rotconv_plan* p, int nq, const uint16_t* w, uint16_t* wt, hipStream_t st);
void launch_p4_fwd_bf16(const rotconv_plan* p, int out_mode, int nq, const uint16_t* x, const uint16_t* wt, void* out_val,
                        uint8_t* out_idx, hipStream_t st);
void launch_p4_combine_bf16(const rotconv_plan* p, const float* pv, const uint8_t* pi, uint16_t* ypool, uint8_t* idx,
                            hipStream_t st);

// input gradient
struct P4BwdGeom {
  int N, Cin, CinPad, H, W, Cout, CoutPad, R, Q, ng;
  int ncig;    // groups of 64 input channels
  int px;      // pixels per lane (2 or 4)
  int nstrip;  // strips of 16 * px pixels per row
  int nw;      // waves (= rows) per workgroup
  int nrb;     // blocks of nw rows
  int ksplit;  // workgroups that share a unit's contraction (each writes an fp32 partial dX); 1 = no split
  int kper;    // weight chunks (16 filters of a bank) per such workgroup
  int units;   // workgroups with work (includes the split)
  int lut;     // routed-gradient table: the contraction runs over the base bank only (Q is 1 then)
  int ncg;     // bf16 table kernel: channel groups of 128 per workgroup (their waves build a K-step's D together)
  int ncigw;   // sets of ncg channel groups
};
bool p4_bwd_lut_choice(const rotconv_plan* p);   // whether the fp32 gradients should use the routed-gradient table
bool p4_bwd_lut(const rotconv_plan* p);          // the plan's setting (contraction over the base bank)
bool p4_bwd_lut16_choice(const rotconv_plan* p); // the same question for the kernels that take bf16 tensors
bool p4_bwd_data_supported(const rotconv_plan* p);
// launch_p4_bwd_data takes the caller's w in place of the packed banks and launch_p4_pack_bwd is not called
bool p4_bwd_data_raw_weights(const rotconv_plan* p);
P4BwdGeom p4_bwd_data_geom(const rotconv_plan* p);
size_t p4_bwd_data_pack_floats(const rotconv_plan* p);
void launch_p4_pack_bwd(const rotconv_plan* p, const float* w, float* wd, hipStream_t st);
// scratch behind the packed bank: the fp32 partial dX of a bank split (0 floats without one)
size_t p4_bwd_data_part_floats(const rotconv_plan* p);
void launch_p4_bwd_data(const rotconv_plan* p, const float* gpool, const uint8_t* idx, const float* wd, float* dx,
                        float* part, hipStream_t st, bool raw_w = false);

// input gradient on bfloat16 tensors (bf16 matrix cores): the forward kernel's row segments and bands with
// the roles of filters and channels swapped
struct P4BwdBfGeom {
  int N, Cin, CIB, H, W, Cout, CoutPad, Q, ng;   // CIB: 16-channel blocks; CoutPad: filters padded to K-steps of 32
  int TY, nbg, units, nwx, nseg, inside;         // as in P4Geom (units include the K split)
  int ksplit, kper;                              // workgroups sharing a unit's K-steps; K-steps per workgroup
  int bank_major;                                // sparse instances: orientations numbered r = 4 q + s instead of r = s Q + q
  int seg_xorg[4], seg_lo[4], seg_hi[4];
};
bool p4_bwd_data_bf16_supported(const rotconv_plan* p);
bool p4_bwd_data_bf16_sparse(const rotconv_plan* p);   // runs the structured-sparse instances (half the matrix instructions)
size_t p4_bwd_data_bf16_pack_bytes(const rotconv_plan* p);
void launch_p4_pack_bwd_bf16(const rotconv_plan* p, const uint16_t* w, uint16_t* wt, hipStream_t st);
size_t p4_bwd_data_bf16_part_bytes(const rotconv_plan* p);
void launch_p4_bwd_data_bf16(const rotconv_plan* p, const uint16_t* gpool, const uint8_t* idx, const uint16_t* wt,
                             uint16_t* dx, float* part, hipStream_t st);

// input gradient on bfloat16 tensors through the routed-gradient table (one contraction with the base bank)
bool p4_bwd_data_bf16_lut_supported(const rotconv_plan* p);
size_t p4_bwd_data_bf16_lut_pack_bytes(const rotconv_plan* p);
size_t p4_bwd_data_bf16_lut_part_bytes(const rotconv_plan* p);
void launch_p4_pack_bwd_bf16_lut(const rotconv_plan* p, const uint16_t* w, uint16_t* wt, hipStream_t st);
void launch_p4_bwd_data_bf16_lut(const rotconv_plan* p, const uint16_t* gpool, const uint8_t* idx, const uint16_t* wt,
                                 uint16_t* dx, float* part, hipStream_t st);

// weight gradient
struct P4BwdWGeom {
  int N, Cin, CinPad, H, W, Cout, CoutPad, Q, ng;
  int ncb;     // 16-channel blocks per wave: 4, or 1 for at most 16 input channels
  int ncig;    // groups of 16 * ncb input channels
  int ncg;     // channel groups per workgroup (their waves build a filter block's D together): 1, 2 or 4
  int ncigw;   // sets of ncg channel groups
  int ncog;    // groups of 4 / ncg (bank, 16-filter block) pairs (one workgroup of 4 waves)
  int nstrip;    // 32-pixel strips per row
  int rows_per;  // rows per range
  int nrange;    // row ranges per image
  int units;     // (image, range, strip) work units
  int splits;    // workgroups per (bank, filter group, channel group); their sums are added in order
  int lut, R;    // routed-gradient table: the sums are those of the base bank (Q is 1 then); orientations
};
bool p4_bwd_weight_supported(const rotconv_plan* p);
P4BwdWGeom p4_bwd_weight_geom(const rotconv_plan* p, bool lut = false, bool share = false);
size_t p4_bwd_weight_ws_floats(const rotconv_plan* p);
void launch_p4_bwd_weight(const rotconv_plan* p, const float* x, const float* gpool, const uint8_t* idx,
                          float* partial, float* dw, hipStream_t st);
// bfloat16 x and gpool (bf16 matrix cores, fp32 partial sums and result); same workspace
bool p4_bwd_weight_bf16_supported(const rotconv_plan* p);
void launch_p4_bwd_weight_bf16(const rotconv_plan* p, const uint16_t* x, const uint16_t* gpool, const uint8_t* idx,
                               float* partial, float* dw, hipStream_t st);

}  // namespace rotconv
