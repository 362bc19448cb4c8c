// Launchers of the HIP kernels (defined in the .hip sources).  Every launcher
// enqueues on `stream` and returns nothing; the API layer checks hipGetLastError.
#pragma once

#include <hip/hip_runtime.h>

#include "rotconv_internal.h"

namespace rotconv {

// Geometry handed to kernels by value.
struct Geom {
  int N, Cin, H, W, Cout, k, kk, R, stride, pad, Ho, Wo, G, ng, B, Q;
  int relu;   // fused pooled forward only: clamp the pooled value at 0 and store idx 255 where it is not positive
};

Geom make_geom(const rotconv_plan* p);

// ---- generic family (any k, stride, pad, R, mode) ----
size_t generic_ws_bytes(const rotconv_plan* p);
int generic_bwdw_splits(const rotconv_plan* p);
// base bank(s) -> R rotated banks [R][Cout][Cin][kk]
void launch_expand_bank(const rotconv_plan* p, const float* w, float* wexp, hipStream_t st);
void launch_fwd_generic(const rotconv_plan* p, const float* x, const float* wexp, float* y, hipStream_t st);
void launch_pool_fwd_generic(const rotconv_plan* p, const float* x, const float* wexp, float* ypool, uint8_t* idx,
                             hipStream_t st);
void launch_bwd_data_generic(const rotconv_plan* p, const float* dy, const float* wexp, float* dx, hipStream_t st);
void launch_pool_bwd_data_generic(const rotconv_plan* p, const float* gpool, const uint8_t* idx, const float* wexp,
                                  float* dx, hipStream_t st);
// partial sums [splits][R][Cout][Cin][kk] into `partial`, then the transposed expansion into dw
void launch_bwd_weight_generic(const rotconv_plan* p, const float* x, const float* dy, const float* gpool,
                               const uint8_t* idx, float* partial, float* dw, hipStream_t st);
// relu: apply the plan's fused activation (the fused forward's fallback through a materialised y); the public
// orient_maxpool_fwd never does
void launch_maxpool_fwd(const rotconv_plan* p, const float* y, float* ypool, uint8_t* idx, hipStream_t st,
                        bool relu = false);
void launch_maxpool_bwd(const rotconv_plan* p, const float* gpool, const uint8_t* idx, float* dy, hipStream_t st);
// average pooling (Eq. 9 / Eq. 11) and the pieces of its fused path
void launch_avgpool_fwd(const rotconv_plan* p, const float* y, float* ypool, hipStream_t st);
void launch_avgpool_bwd(const rotconv_plan* p, const float* gpool, float* dy, hipStream_t st);
void launch_avgpool_fwd_bf16(const rotconv_plan* p, const uint16_t* y, uint16_t* ypool, hipStream_t st);
void launch_avgpool_bwd_bf16(const rotconv_plan* p, const uint16_t* gpool, uint16_t* dy, hipStream_t st);
// wavg[(co*ng+g)][ci][t] = (1/G) sum_{r mod ng == g} wexp[r][co][ci][t]
void launch_avg_bank(const rotconv_plan* p, const float* wexp, float* wavg, hipStream_t st);
// its adjoint: rep[r][co][ci][t] = dwavg[(co*ng + r mod ng)][ci][t] / G, then the transposed expansion into dw
void launch_avg_bank_bwd(const rotconv_plan* p, const float* dwavg, float* rep, float* dw, hipStream_t st);
void launch_fill_u8(uint8_t* p, size_t n, uint8_t v, hipStream_t st);
void launch_maxpool_fwd_bf16(const rotconv_plan* p, const uint16_t* y, uint16_t* ypool, uint8_t* idx, hipStream_t st);
void launch_maxpool_bwd_bf16(const rotconv_plan* p, const uint16_t* gpool, const uint8_t* idx, uint16_t* dy,
                             hipStream_t st);

}  // namespace rotconv
