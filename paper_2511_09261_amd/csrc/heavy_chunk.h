// Chunked pre-reduction of rows with very many neighbours (bf16 features): the work of ONE
// workgroup on ONE chunk, as a device function, so that the launch that precedes an
// aggregation can carry the chunks as extra workgroups instead of a launch of their own.
//   partial[ch, :] = sum over the entries e of chunk ch of  A_hat value(e) * x(column(e), :)
// in fp32.  Lane group grp (the lanes that share one 16-byte slice per lane of a feature
// row) takes entries grp, grp + G, ..., four loads in flight; the G group sums are added in
// order.  `red` is kBlock * 8 floats of LDS.  Contains a workgroup barrier.
#pragma once

#include "bf16_common.h"
#include "device_utils.h"
#include "gco_internal.h"

namespace gco {

// x(j, :) = X[j, :]
template <int D>
struct ChunkPlainRows {
  const bf16_t* X;
  __device__ __forceinline__ void add(int j, int c0, float val, float (&acc)[8]) const {
    float v[8];
    unpack8(*reinterpret_cast<const uint4*>(X + static_cast<size_t>(j) * D + c0), v);
#pragma unroll
    for (int y = 0; y < 8; ++y) acc[y] = fmaf(val, v[y], acc[y]);
  }
};

// x(j, c) = bf16(g_t[j] * w[c]) where H[j, c] > 0, else 0: the rows of dL/dZ of the last
// hidden layer, formed on the fly exactly as the kernel that stores them forms them.
template <int D>
struct ChunkLastLayerRows {
  const bf16_t* H;
  const float* g_t;
  float w[8];  // the scalar layer's weights of this lane's eight features
  __device__ __forceinline__ void add(int j, int c0, float val, float (&acc)[8]) const {
    float hv[8];
    unpack8(*reinterpret_cast<const uint4*>(H + static_cast<size_t>(j) * D + c0), hv);
    const float gt = g_t[j];
#pragma unroll
    for (int y = 0; y < 8; ++y) {
      const float x = hv[y] > 0.f ? bf16_to_f32(f32_to_bf16(gt * w[y])) : 0.f;
      acc[y] = fmaf(val, x, acc[y]);
    }
  }
};

template <int D, class Rows>
__device__ __forceinline__ void reduce_chunk(const GraphView& g, const Rows& rows, float* __restrict__ partial,
                                             int ch, float* red) {
  constexpr int LPR = D / 8;       // lanes per feature row (16 bytes each)
  constexpr int G = kBlock / LPR;  // lane groups per workgroup
  const int tid = threadIdx.x;
  const int grp = tid / LPR, c0 = (tid % LPR) * 8;
  float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const int eb = g.chunk_end[ch];
  for (int e = g.chunk_begin[ch] + grp; e < eb; e += 4 * G) {
    int2 en[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) en[x] = e + x * G < eb ? g.ent[e + x * G] : make_int2(-1, 0);
#pragma unroll
    for (int x = 0; x < 4; ++x)
      if (en[x].x >= 0) rows.add(en[x].x, c0, __int_as_float(en[x].y), a8);
  }
#pragma unroll
  for (int x = 0; x < 8; ++x) red[grp * D + c0 + x] = a8[x];
  __syncthreads();
  if (tid < D) {
    float sum = 0.f;
    for (int gq = 0; gq < G; ++gq) sum += red[gq * D + tid];
    partial[static_cast<size_t>(ch) * D + tid] = sum;
  }
}

}  // namespace gco
