// Declarations of the matrix-multiply + scatter family (any k, stride, pad; fp32).
#pragma once

#include <hip/hip_runtime.h>

#include "rotconv_internal.h"

namespace rotconv {

bool gs_wanted(const rotconv_plan* p);       // the family pays off for this plan's shape
size_t gs_chunk_budget(const rotconv_plan* p);                    // bytes of products held at once (default 512 MiB)
size_t gs_ws_bytes(const rotconv_plan* p);   // packed banks, products / routed gradients of a few images, partial sums
void launch_gs_fwd(const rotconv_plan* p, const float* x, const float* w, float* y, void* ws, hipStream_t st);
void launch_gs_pool_fwd(const rotconv_plan* p, const float* x, const float* w, float* ypool, uint8_t* idx, void* ws,
                        hipStream_t st);   // applies the plan's fused activation
void launch_gs_bwd_data(const rotconv_plan* p, const float* dy, const float* w, float* dx, void* ws, hipStream_t st);
void launch_gs_pool_bwd_data(const rotconv_plan* p, const float* gpool, const uint8_t* idx, const float* w, float* dx,
                             void* ws, hipStream_t st);
void launch_gs_bwd_weight(const rotconv_plan* p, const float* x, const float* dy, float* dw, void* ws, hipStream_t st);
void launch_gs_pool_bwd_weight(const rotconv_plan* p, const float* x, const float* gpool, const uint8_t* idx, float* dw,
                               void* ws, hipStream_t st);

}  // namespace rotconv
