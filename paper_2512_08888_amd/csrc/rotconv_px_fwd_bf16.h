// Pooled forward on bf16 tensors with the filters on the matrix instruction's M side and sixteen pixels on its N side.
#pragma once

#include <hip/hip_runtime.h>

#include "rotconv_internal.h"

namespace rotconv {

bool px_fwd_bf16_supported(const rotconv_plan* p);
size_t px_fwd_bf16_pack_bytes(const rotconv_plan* p);
// wt: px_fwd_bf16_pack_bytes(p) bytes of scratch for the packed banks (16-byte aligned)
void launch_px_fwd_bf16(const rotconv_plan* p, const uint16_t* x, const uint16_t* w, uint16_t* ypool, uint8_t* idx,
                        uint16_t* wt, hipStream_t st);

}  // namespace rotconv
