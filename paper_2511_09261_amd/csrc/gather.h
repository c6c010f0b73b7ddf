// Device code shared by the wide (feature-matrix) kernels: the sources of
// gathered rows and the fixed-order row gather.
#pragma once

#include "device_utils.h"
#include "gco_internal.h"

namespace gco {

// ---------------------------------------------------------------------------
// Sources of gathered rows
// ---------------------------------------------------------------------------

// v = sb[j] * X[j, c0 .. c0+VEC)
template <typename T, int D>
struct PlainSrc {
  static constexpr int VEC = Store<T>::VEC;
  const T* X;
  const float* sb;
  __device__ __forceinline__ void set_part(int, int) {}
  __device__ __forceinline__ void load(int j, int c0, float (&v)[VEC]) const {
    Store<T>::load(X + static_cast<size_t>(j) * D + c0, v);
    const float s = sb[j];
#pragma unroll
    for (int x = 0; x < VEC; ++x) v[x] *= s;
  }
};

// Gradient of the last hidden layer's pre-activation, formed on the fly:
// v = sb[j] * g_t[j] * w_out[c] * [H[j, c] > 0]
template <typename T, int D>
struct LastSrc {
  static constexpr int VEC = Store<T>::VEC;
  const T* H;
  const float* sb;
  const float* g_t;
  const float* w_out;  // [Pw, D]
  int wout_stride;
  float w[VEC];
  __device__ __forceinline__ void set_part(int k, int c0) {
#pragma unroll
    for (int x = 0; x < VEC; ++x) w[x] = w_out[static_cast<size_t>(k) * wout_stride + c0 + x];
  }
  __device__ __forceinline__ void load(int j, int c0, float (&v)[VEC]) const {
    Store<T>::load(H + static_cast<size_t>(j) * D + c0, v);
    const float s = sb[j] * g_t[j];
#pragma unroll
    for (int x = 0; x < VEC; ++x) v[x] = v[x] > 0.f ? s * w[x] : 0.f;
  }
};

// acc += sum over entries e0, e0+stride, ... < e1 of src(col[e]); four rows in flight.
template <class Src>
__device__ __forceinline__ void gather_range(const Src& src, const int* __restrict__ col, int e0,
                                             int e1, int stride, int c0,
                                             float (&acc)[Src::VEC]) {
  constexpr int VEC = Src::VEC;
  int e = e0;
  for (; e + 3 * stride < e1; e += 4 * stride) {
    const int j0 = col[e], j1 = col[e + stride], j2 = col[e + 2 * stride], j3 = col[e + 3 * stride];
    float v0[VEC], v1[VEC], v2[VEC], v3[VEC];
    src.load(j0, c0, v0);
    src.load(j1, c0, v1);
    src.load(j2, c0, v2);
    src.load(j3, c0, v3);
#pragma unroll
    for (int x = 0; x < VEC; ++x) acc[x] = (((acc[x] + v0[x]) + v1[x]) + v2[x]) + v3[x];
  }
  for (; e < e1; e += stride) {
    float v0[VEC];
    src.load(col[e], c0, v0);
#pragma unroll
    for (int x = 0; x < VEC; ++x) acc[x] += v0[x];
  }
}

// Phase 1 of the wide kernels: row r of the tile becomes
//   sa_i * ( src(i) + sum_{j in N(i)} src(j) ),  i = row0 + r,
// handed to `sink` (put_vec: VEC consecutive columns of a row; put_one: a single
// element); rows nrows..kTileRows are handed zeros.  Short rows are summed by
// one lane group, rows longer than kLightMax by the whole workgroup in a second
// pass, and pre-reduced rows take their chunk partials.
// LDS: red [kBlock * VEC] floats, hlist [kTileRows + 1] ints.  Ends with a barrier.
template <typename T, int D, class Src, class Sink>
__device__ void aggregate_tile(const GraphView& g, const Src& src, const Sink& sink, int row0,
                               int nrows, float* red, int* hlist,
                               const float* __restrict__ heavy_partial) {
  constexpr int VEC = Store<T>::VEC;
  constexpr int LPR = D / VEC;        // lanes per feature row
  constexpr int G = kBlock / LPR;     // lane groups per workgroup
  const int tid = threadIdx.x;
  const int grp = tid / LPR;
  const int c0 = (tid % LPR) * VEC;
  if (tid == 0) hlist[0] = 0;
  __syncthreads();
  for (int r = grp; r < kTileRows; r += G) {
    float acc[VEC];
    if (r >= nrows) {
#pragma unroll
      for (int x = 0; x < VEC; ++x) acc[x] = 0.f;
      sink.template put_vec<VEC>(r, c0, acc);
      continue;
    }
    const int i = row0 + r;
    const int e0 = g.rowptr[i], e1 = g.rowptr[i + 1];
    const int h = g.num_heavy > 0 ? g.heavy_of_row[i] : -1;
    if (h < 0 && e1 - e0 > kLightMax) {
      if (tid % LPR == 0) {
        const int q = atomicAdd(&hlist[0], 1);
        hlist[1 + q] = r;
      }
      continue;
    }
    src.load(i, c0, acc);  // the self loop of A + I
    if (h >= 0) {
      for (int ch = g.heavy_chunk_ptr[h]; ch < g.heavy_chunk_ptr[h + 1]; ++ch) {
        const float4* pp = reinterpret_cast<const float4*>(heavy_partial + static_cast<size_t>(ch) * D + c0);
#pragma unroll
        for (int x = 0; x < VEC; x += 4) {
          const float4 q4 = pp[x / 4];
          acc[x] += q4.x; acc[x + 1] += q4.y; acc[x + 2] += q4.z; acc[x + 3] += q4.w;
        }
      }
    } else {
      gather_range(src, g.col, e0, e1, 1, c0, acc);
    }
    const float sa = g.sa[i];
#pragma unroll
    for (int x = 0; x < VEC; ++x) acc[x] *= sa;
    sink.template put_vec<VEC>(r, c0, acc);
  }
  __syncthreads();
  const int nh = hlist[0];
  for (int q = 0; q < nh; ++q) {
    const int r = hlist[1 + q];
    const int i = row0 + r;
    const int e0 = g.rowptr[i], e1 = g.rowptr[i + 1];
    float acc[VEC];
    if (grp == 0) {
      src.load(i, c0, acc);
    } else {
#pragma unroll
      for (int x = 0; x < VEC; ++x) acc[x] = 0.f;
    }
    gather_range(src, g.col, e0 + grp, e1, G, c0, acc);
#pragma unroll
    for (int x = 0; x < VEC; ++x) red[grp * D + c0 + x] = acc[x];
    __syncthreads();
    if (tid < D) {
      float s = 0.f;
      for (int gq = 0; gq < G; ++gq) s += red[gq * D + tid];
      sink.put_one(r, tid, g.sa[i] * s);
    }
    __syncthreads();
  }
}

// Chunked pre-reduction of very long rows: partial[c, :] = sum_{e in chunk c} src(col[e]).
template <typename T, int D, class Src>
__global__ __launch_bounds__(kBlock) void heavy_wide_kernel(GraphView g, Src src, float* partial) {
  constexpr int VEC = Store<T>::VEC;
  constexpr int LPR = D / VEC;
  constexpr int G = kBlock / LPR;
  __shared__ float red[kBlock * VEC];
  const int ch = blockIdx.x;
  const int tid = threadIdx.x;
  const int grp = tid / LPR;
  const int c0 = (tid % LPR) * VEC;
  if (g.chunk_part[ch] < 0) return;  // the row's subgraph sits out
  src.set_part(g.chunk_part[ch], c0);
  float acc[VEC];
#pragma unroll
  for (int x = 0; x < VEC; ++x) acc[x] = 0.f;
  gather_range(src, g.col, g.chunk_begin[ch] + grp, g.chunk_end[ch], G, c0, acc);
#pragma unroll
  for (int x = 0; x < VEC; ++x) red[grp * D + c0 + x] = acc[x];
  __syncthreads();
  if (tid < D) {
    float s = 0.f;
    for (int gq = 0; gq < G; ++gq) s += red[gq * D + tid];
    partial[static_cast<size_t>(ch) * D + tid] = s;
  }
}

}  // namespace gco
