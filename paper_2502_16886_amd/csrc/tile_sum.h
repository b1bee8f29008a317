// Sum of the squared scores of one 32-position tile, in fp64.  Lanes 0..31 of a wavefront hold
// one score each (0 for positions past the sequence end).  The butterfly order is fixed, so
// every kernel that forms a tile sum produces the same bits for the same scores.
#pragma once

#include <hip/hip_runtime.h>

namespace rfkv {

constexpr int kTileKeys = 32;

__device__ __forceinline__ double tile_sum_sq(float score, int lane) {
  double v = lane < 32 ? (double)score * (double)score : 0.0;
#pragma unroll
  for (int d = 16; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  return v;     // valid in lanes 0..31
}

}  // namespace rfkv
