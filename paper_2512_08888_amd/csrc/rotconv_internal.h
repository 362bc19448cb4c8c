// Internal declarations shared by the host code and the HIP kernels of the
// rotation-convolution library.  Not part of the C ABI.
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "rotconv.h"

namespace rotconv {

// One non-zero of the expansion map: W^(r)[dst tap] += coef * w[src], src = b*k*k + u.
constexpr int kMaxNnz = 4;

struct HostTables {
  // Orientation structure (Sec. III-D): theta_r = 90*quarter[r] + phi[bank[r]].
  int Q = 0;
  std::vector<int> bank_of_r, quarter_of_r;
  std::vector<double> phi_deg;  // per first-quadrant bank
  std::vector<int> mirrored;    // per bank: built from the left-right mirrored base filter (P4M mode)
  // Forward expansion, one row per (r, dst tap): up to kMaxNnz (src, coef) pairs, src = -1 unused.
  std::vector<int32_t> exp_src;  // [R*kk*kMaxNnz]
  std::vector<float> exp_coef;   // [R*kk*kMaxNnz]
  // The same coefficients as computed (fp64): bf16 plans form the banks they multiply with in fp64 and round the
  // result once, so that the rounding does not depend on fp32 intermediate error.
  std::vector<double> exp_coef64, fq_coef64;
  // 3x3 plans: the first-quadrant expansion as dense fp64 matrices [Q][9 taps][B * 9 source taps] (the bf16 bank
  // packing multiplies with wave-uniform coefficients)
  std::vector<double> fq_dense64;
  // Transposed expansion in CSR form, one row per base element (b, u):
  // dw[b][u] = sum over entries e in row: coef[e] * dW^(r_e)[t_e], col = r*kk + t.
  std::vector<int32_t> tr_ptr;   // [B*kk + 1]
  std::vector<int32_t> tr_col;
  std::vector<float> tr_coef;
  // First-quadrant expansion (base -> Q banks, before any quarter turn), same row format
  // as exp_*, one row per (q, dst tap); and its transpose in CSR form (col = q*kk + t).
  std::vector<int32_t> fq_src;
  std::vector<float> fq_coef;
  std::vector<int32_t> fqt_ptr, fqt_col;
  std::vector<float> fqt_coef;
  // Quarter-turn tap permutation: turn_tap[s*kk + u] = index of the tap where base tap u
  // sits after s quarter turns (Eq. 8: (m',n') = R_s(m,n)).
  std::vector<int32_t> turn_tap;  // [4*kk]
  // 3x3 plans: [B base banks][9 neighbour offsets][R + 1][12] routed-gradient coefficients (see rotconv_host.cpp)
  std::vector<float> lut_bwd;
  // forward on base products: [Q][9 taps][4] coefficients of a bank's products in terms of the base products, in
  // the order of the compiled source pattern (empty unless the plan uses that kernel)
  std::vector<float> fwd_base_coef;
};

struct DeviceTables {
  int device = -1;
  int32_t* exp_src = nullptr;
  float* exp_coef = nullptr;
  double* exp_coef64 = nullptr;  // bf16 plans only (one element otherwise)
  double* fq_coef64 = nullptr;
  double* fq_dense64 = nullptr;  // bf16 plans only (one element otherwise)
  int32_t* tr_ptr = nullptr;
  int32_t* tr_col = nullptr;
  float* tr_coef = nullptr;
  int32_t* fq_src = nullptr;
  float* fq_coef = nullptr;
  int32_t* fqt_ptr = nullptr;
  int32_t* fqt_col = nullptr;
  float* fqt_coef = nullptr;
  int32_t* rot_of = nullptr;  // [Q*4] orientation index r of (bank q, quarter s), -1 if absent
  int32_t* rq_of_r = nullptr;   // [R] bank * 4 + quarter turn of orientation r
  int32_t* turn_tap = nullptr;  // [4*kk] tap position of base tap u after s quarter turns
  float* lut_bwd = nullptr;     // HostTables::lut_bwd (one element if the plan has none)
  float* fwd_base_coef = nullptr;   // HostTables::fwd_base_coef (one element if the plan has none)
};

}  // namespace rotconv

struct rotconv_plan {
  rotconv_desc d;               // angles_deg is redirected to `angles`
  rotconv_plan_options opt{};   // tuning switches (all zero: automatic); the plans a plan owns inherit them
  std::vector<double> angles;
  int B = 1, G = 1, ng = 1, Ho = 0, Wo = 0, kk = 0;
  rotconv::HostTables host;
  std::vector<int32_t> rot_of;  // [Q*4]
  rotconv::DeviceTables dev;    // uploaded on first launch
  size_t ws_bytes = 0;          // what the caller must provide
  size_t ws_inner = 0;          // what the fp32 kernels need (== ws_bytes for fp32 plans)
  size_t n_x = 0, n_w = 0, n_yp = 0, n_yu = 0;   // elements of input, base weights, pooled and unpooled output
  // kernel selection per pass (0 fwd, 1 bwd_data, 2 bwd_weight)
  int fast[3] = {0, 0, 0};
  // bf16 plans: the pass has a kernel that reads and writes bfloat16 directly (bf16 matrix cores); the
  // other passes run the fp32 kernels on widened copies
  int native16[3] = {0, 0, 0};
  int bwdw_splits = 1;          // pixel splits of the generic weight-gradient kernel
  size_t gs_chunk_bytes = (size_t)512 << 20;   // that family holds the products of as many images as fit this
  int gs = 0;                   // passes without a register-resident kernel run the matrix-multiply + scatter family
  int bwd_lut = 0;              // fast fp32 gradients: routed-gradient table, contraction over the base bank only
  int bwd_lut16[3] = {0, 0, 0}; // bf16 gradient kernels ([1] input, [2] weight gradient): the same table, D rounded to bf16 once
  int fwd_base = 0;             // fast fp32 pooled forward: products of the base bank only, banks combined on the vector ALU
  int fwd_base_cls = 0;         // its banks' classes (two bits per bank)
  int direct[3] = {0, 0, 0};    // the pass runs the vector-ALU kernel of layers with at most four input channels
  int px16 = 0;                 // bf16 pooled forward: the kernel with a lane per pixel column (filters on M)
  int fwd_csplit[2] = {1, 1};   // fast forward: channel splits for the unpooled / the pooled output (1: none)
  // Average pooling (Eq. 9 / Eq. 11): the fused calls run one ordinary convolution (this R = 1 plan with
  // Cout * R/G filters) on the group-averaged bank.  Owned by the parent.
  rotconv_plan* avg_child = nullptr;
  // Row widths the matrix-core kernels do not take (odd, not a multiple of 4 for the weight gradient, ...): the
  // fused calls and rotconv_fwd run this plan of the same layer on zero-padded rows (width a multiple of 8) through
  // staging copies; columns beyond W hold zeros / idx 255, which is what the convolution's own padding supplies.
  // pad_use[pass]: the pass is faster there.  Owned by the parent.
  rotconv_plan* pad_child = nullptr;
  int pad_use[3] = {0, 0, 0};
};

namespace rotconv {

// Host logic (rotconv_host.cpp).
int validate_and_build(const rotconv_desc* desc, rotconv_plan** out);

// Kernel launchers (HIP sources).  All return a rotconv_status.
int ensure_device_tables(rotconv_plan* plan);
void free_device_tables(rotconv_plan* plan);

}  // namespace rotconv
