// Helpers shared by the bf16 layer kernels: matrix-core fragment types and the
// packing of eight fp32 values into 16 bytes of bf16 and back.
#pragma once

#include "device_utils.h"
#include "gco_internal.h"

namespace gco {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ bf16x8 as_frag(const uint4& u) {
  bf16x8 v;
  __builtin_memcpy(&v, &u, 16);
  return v;
}

__device__ __forceinline__ uint4 pack8(const float (&v)[8]) {
  uint4 x;
  x.x = f32x2_to_bf16x2(v[0], v[1]);
  x.y = f32x2_to_bf16x2(v[2], v[3]);
  x.z = f32x2_to_bf16x2(v[4], v[5]);
  x.w = f32x2_to_bf16x2(v[6], v[7]);
  return x;
}

__device__ __forceinline__ void unpack8(const uint4& x, float (&v)[8]) {
  v[0] = __uint_as_float(x.x << 16); v[1] = __uint_as_float(x.x & 0xffff0000u);
  v[2] = __uint_as_float(x.y << 16); v[3] = __uint_as_float(x.y & 0xffff0000u);
  v[4] = __uint_as_float(x.z << 16); v[5] = __uint_as_float(x.z & 0xffff0000u);
  v[6] = __uint_as_float(x.w << 16); v[7] = __uint_as_float(x.w & 0xffff0000u);
}

// Index of row i in the ascending list of pre-reduced rows (i must be in it).
__device__ __forceinline__ int find_heavy(const GraphView& g, int i) {
  int lo = 0, hi = g.num_heavy - 1;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (g.heavy_rows[mid] < i) lo = mid + 1; else hi = mid;
  }
  return lo;
}

}  // namespace gco
