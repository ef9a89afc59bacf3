// Block-wide exclusive scan of one uint32 per thread (wave64 shuffles + one LDS hop).
#pragma once

#include "common.h"

namespace hctr {

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    uint32_t t = __shfl_up(v, d);
    if (lane >= d) v += t;
  }
  return v;
}

// Exclusive scan over a block of NT threads; *block_total gets the sum.  lds holds NT/64 + 1 words
// and may be reused by the caller as soon as the call returns.
template <int NT>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* lds, uint32_t* block_total) {
  constexpr int NW = NT / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t inc = wave_inclusive_scan(v);
  if (lane == 63) lds[wave] = inc;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t run = 0;
    for (int w = 0; w < NW; ++w) {
      uint32_t t = lds[w];
      lds[w] = run;
      run += t;
    }
    lds[NW] = run;
  }
  __syncthreads();
  uint32_t res = inc - v + lds[wave];
  *block_total = lds[NW];
  __syncthreads();
  return res;
}

}  // namespace hctr
