// Quarter-turn tap geometry shared by the fast forward kernels (paper Eq. 8).
#pragma once

namespace rotconv {

// Row / column of base tap u inside the 3x3 filter turned by s quarter turns.
__device__ __host__ constexpr int tap_i(int s, int u) {
  return s == 0 ? u / 3 : s == 1 ? 2 - u % 3 : s == 2 ? 2 - u / 3 : u % 3;
}
__device__ __host__ constexpr int tap_j(int s, int u) {
  return s == 0 ? u % 3 : s == 1 ? u / 3 : s == 2 ? 2 - u % 3 : 2 - u / 3;
}
// Index of non-centre tap u in the 8-entry edge exchange arrays.
__device__ __host__ constexpr int edge_slot(int u) { return u < 4 ? u : u - 1; }

}  // namespace rotconv
