// Helpers of the row kernels (layer norm, softmax): one wave owns a row of FP16 values and keeps it in
// registers; reductions over the row are cross-lane butterflies with a fixed order of operations.
#pragma once

#include "us_device.h"

namespace us {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = __builtin_fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

// A row of n FP16 values as NCH chunks of 8 per lane: chunk k of lane l covers columns (k*64 + l)*8 .. +7.
template <int NCH>
struct RowRegs {
  v8h v[NCH];
  __device__ __forceinline__ void load(const _Float16* row, int n, int lane) {
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
      const int col = (k * 64 + lane) * 8;
      if (col < n) v[k] = *reinterpret_cast<const v8h*>(row + col);
      else v[k] = v8h{0, 0, 0, 0, 0, 0, 0, 0};
    }
  }
};

}  // namespace us
