// Forward (and weight gradient) of layers with at most four input channels on the vector ALU.
#pragma once

#include <hip/hip_runtime.h>

#include "rotconv_internal.h"

namespace rotconv {

bool direct_fwd_supported(const rotconv_plan* p);
size_t direct_fwd_pack_floats(const rotconv_plan* p);
// x, ypool: float for fp32 plans, bfloat16 for bf16 plans
void launch_direct_fwd(const rotconv_plan* p, const void* x, const void* w, void* ypool, uint8_t* idx, float* wb,
                       hipStream_t st);

// weight gradient (single-bank layers): `part` holds direct_bwd_weight_ws_floats(p) floats of partial sums
bool direct_bwd_weight_supported(const rotconv_plan* p);
size_t direct_bwd_weight_ws_floats(const rotconv_plan* p);
void launch_direct_bwd_weight(const rotconv_plan* p, const void* x, const void* gpool, const uint8_t* idx, float* part,
                              float* dw, hipStream_t st);

}  // namespace rotconv
