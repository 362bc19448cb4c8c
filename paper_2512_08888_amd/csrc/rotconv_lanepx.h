// Device helpers of the kernels in which a lane owns one pixel column and reads its neighbours' products through lane
// shifts inside the placement additions (paper Eq. 8): the tap geometry, the placement block, maxima, stores.
#pragma once

#include <hip/hip_runtime.h>

#include "rotconv_bf16.h"
#include "rotconv_p4_taps.h"

namespace rotconv {
namespace {

// Stores at a wave-uniform base plus the lane's 32-bit byte offset (the address form that needs no per-lane 64-bit
// arithmetic; written out because the compiler folds the two into a per-lane pointer and adds per store).
__device__ __forceinline__ void st_at(float* base, unsigned byte_off, float v) {
  asm volatile("global_store_dword %0, %1, %2" ::"v"(byte_off), "v"(v), "s"(base) : "memory");
}
__device__ __forceinline__ void st_at(uint16_t* base, unsigned byte_off, float v) {
  const unsigned h = f32_to_bf16(v);
  asm volatile("global_store_short %0, %1, %2" ::"v"(byte_off), "v"(h), "s"(base) : "memory");
}
__device__ __forceinline__ void st_at(uint8_t* base, unsigned byte_off, int v) {
  asm volatile("global_store_byte %0, %1, %2" ::"v"(byte_off), "v"(v), "s"(base) : "memory");
}

// Base tap that sits at row i, column j of the 3 x 3 filter after s quarter turns (the inverse of tap_i / tap_j).
constexpr int kTapAt[4][3][3] = {{{0, 1, 2}, {3, 4, 5}, {6, 7, 8}},
                                 {{2, 5, 8}, {1, 4, 7}, {0, 3, 6}},
                                 {{8, 7, 6}, {5, 4, 3}, {2, 1, 0}},
                                 {{6, 3, 0}, {7, 4, 1}, {8, 5, 2}}};
constexpr bool tap_table_ok() {
  for (int s = 0; s < 4; ++s)
    for (int u = 0; u < 9; ++u)
      if (kTapAt[s][tap_i(s, u)][tap_j(s, u)] != u) return false;
  return true;
}
static_assert(tap_table_ok(), "kTapAt is the inverse of tap_i / tap_j");

// Placement of one product row for the four quarter turns of a bank (Eq. 8).  P[u]: the lane's nine products of row h.
// Row 2 of the turned filter completes output row h-1 (o = A + ...), row 1 continues output row h (A = B + ...), row 0
// starts output row h+1 (B = ...); column 0 takes the product of the lane to the left (DPP_L: a shift right by one lane), column 2 the
// one to the right (DPP_R), read by the addition itself.  The operand numbers below are kTapAt[s][i][j] + 12.  Written
// as one block so that the order is fixed: the four orientations' chains are interleaved, and the first four
// instructions read no lane-shifted operand, so a shifted read is at least two instructions behind the write of any of
// its registers (the wait the hardware asks for between a vector write and a DPP read).
#define ROTCONV_PLACE_ROW(NAME, DPP_L, DPP_R)                                                                        \
__device__ __forceinline__ void NAME(const float (&P)[9], float (&A)[4], float (&B)[4], float (&o)[4]) {             \
  asm volatile(                                                                                                        \
      "v_add_f32 %0, %19, %4\n\t"                                                                                     \
      "v_add_f32 %1, %15, %5\n\t"                                                                                     \
      "v_add_f32 %2, %13, %6\n\t"                                                                                     \
      "v_add_f32 %3, %17, %7\n\t"                                                                                     \
      "v_add_f32_dpp %0, %18, %0 " DPP_L                                                                              \
      "v_add_f32_dpp %1, %12, %1 " DPP_L                                                                              \
      "v_add_f32_dpp %2, %14, %2 " DPP_L                                                                              \
      "v_add_f32_dpp %3, %20, %3 " DPP_L                                                                              \
      "v_add_f32_dpp %0, %20, %0 " DPP_R                                                                              \
      "v_add_f32_dpp %1, %18, %1 " DPP_R                                                                              \
      "v_add_f32_dpp %2, %12, %2 " DPP_R                                                                              \
      "v_add_f32_dpp %3, %14, %3 " DPP_R                                                                              \
      "v_add_f32 %4, %16, %8\n\t"                                                                                     \
      "v_add_f32 %5, %16, %9\n\t"                                                                                     \
      "v_add_f32 %6, %16, %10\n\t"                                                                                    \
      "v_add_f32 %7, %16, %11\n\t"                                                                                    \
      "v_add_f32_dpp %4, %15, %4 " DPP_L                                                                              \
      "v_add_f32_dpp %5, %13, %5 " DPP_L                                                                              \
      "v_add_f32_dpp %6, %17, %6 " DPP_L                                                                              \
      "v_add_f32_dpp %7, %19, %7 " DPP_L                                                                              \
      "v_add_f32_dpp %4, %17, %4 " DPP_R                                                                              \
      "v_add_f32_dpp %5, %19, %5 " DPP_R                                                                              \
      "v_add_f32_dpp %6, %15, %6 " DPP_R                                                                              \
      "v_add_f32_dpp %7, %13, %7 " DPP_R                                                                              \
      "v_add_f32_dpp %8, %12, %13 " DPP_L                                                                             \
      "v_add_f32_dpp %9, %14, %17 " DPP_L                                                                             \
      "v_add_f32_dpp %10, %20, %19 " DPP_L                                                                            \
      "v_add_f32_dpp %11, %18, %15 " DPP_L                                                                            \
      "v_add_f32_dpp %8, %14, %8 " DPP_R                                                                              \
      "v_add_f32_dpp %9, %20, %9 " DPP_R                                                                              \
      "v_add_f32_dpp %10, %18, %10 " DPP_R                                                                            \
      "v_add_f32_dpp %11, %12, %11 " DPP_R                                                                            \
      : "=&v"(o[0]), "=&v"(o[1]), "=&v"(o[2]), "=&v"(o[3]), "+v"(A[0]), "+v"(A[1]), "+v"(A[2]), "+v"(A[3]), "+v"(B[0]),\
        "+v"(B[1]), "+v"(B[2]), "+v"(B[3])                                                                            \
      : "v"(P[0]), "v"(P[1]), "v"(P[2]), "v"(P[3]), "v"(P[4]), "v"(P[5]), "v"(P[6]), "v"(P[7]), "v"(P[8]));           \
}
// whole-wave shifts: 64 lanes = 64 consecutive columns; shifts inside a 16-lane row: 16 lanes = 16 consecutive columns
ROTCONV_PLACE_ROW(place_row, "wave_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t",
                  "wave_shl:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t")
ROTCONV_PLACE_ROW(place_row16, "row_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t",
                  "row_shl:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t")
#undef ROTCONV_PLACE_ROW

// maxima without the canonicalising self-maximum the compiler puts in front of fmaxf (NaN inputs are undefined here)
__device__ __forceinline__ float max2(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}


}  // namespace
}  // namespace rotconv
