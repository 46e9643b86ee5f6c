// Shared by the grouped-FFN kernel files: persistent work distribution.
#pragma once
#include "kernels.h"

namespace mp {

// Persistent work distribution that keeps neighbouring work items on one XCD.
// Workgroups are handed to the 8 XCDs round-robin by workgroup id, and each XCD
// has its own L2.  Workgroup b therefore serves XCD b % 8 and walks a contiguous
// eighth of the item list together with the other workgroups of that XCD, so
// the tiles that share an activation tile or a sub-expert's weights meet in one L2.
constexpr int N_XCD = 8;
struct ItemRange {
  int begin, end, step;
};
__device__ __forceinline__ ItemRange xcd_items(int total) {
  const int xcd = blockIdx.x % N_XCD, slot = blockIdx.x / N_XCD;
  const int per = gridDim.x / N_XCD;  // the grid is a multiple of N_XCD
  const int chunk = (total + N_XCD - 1) / N_XCD;
  ItemRange r;
  r.begin = min(total, xcd * chunk) + slot;
  r.end = min(total, (xcd + 1) * chunk);
  r.step = per;
  return r;
}

inline int persistent_grid(long max_items, int per_cu) {  // a multiple of N_XCD
  long g = (long)num_cus() * per_cu;
  if (g > max_items) g = max_items;
  if (g < 1) g = 1;
  return (int)((g + N_XCD - 1) / N_XCD * N_XCD);
}

// bf16 kernels (ffn_bf16.hip)
hipError_t launch_gate_up_bf16(const uint16_t* x, const uint16_t* w_gu, const int32_t* sorted_pair,
                               const MTile* tiles, int32_t* hdr, uint16_t* h, int T, int d,
                               int Is, int k_max, int max_mtiles, hipStream_t s);
hipError_t launch_down_bf16(const uint16_t* h, const uint16_t* w_dn, const MTile* tiles,
                            int32_t* hdr, uint16_t* y, int d, int Is, int max_mtiles,
                            hipStream_t s);

}  // namespace mp
