// Training-step kernels for gfx950: fused aggregate+transform layers (Eq. 3),
// read-out (Eq. 4), loss and its gradient (Eq. 5), backward passes and Adam.
//
// Work decomposition.  Nodes are stored subgraph by subgraph.  A workgroup is
// bound to one subgraph k (so its weight matrix W^k sits in LDS once) and walks
// that subgraph's row tiles s, s+S, s+2S, ...  Within a tile:
//   phase 1  gather: A_hat rows times the feature matrix, fp32 accumulation,
//            result left in an LDS tile.  Short rows are taken by small lane
//            groups (one 16-byte slice of the feature row per lane), long rows by
//            the whole workgroup, very long rows come pre-reduced in chunks;
//   phase 2  dense transform of the LDS tile with W^k and the fused epilogue.
// Every sum is taken in an order fixed by the launch shape, so results are
// bit-identical from run to run.
#include "device_utils.h"
#include "gather.h"
#include "gco_internal.h"
#include "heavy_chunk.h"

namespace gco {
namespace {

constexpr int R = kTileRows;

template <int D>
struct Geo {
  static constexpr int LD = D + 4;  // LDS row pitch in floats (keeps 16-byte alignment)
};

// Where the fp32 kernels leave the gathered rows: an fp32 LDS tile [R][LD].
template <int D>
struct TileSink {
  float* tile;
  template <int VEC>
  __device__ __forceinline__ void put_vec(int r, int c0, const float (&v)[VEC]) const {
#pragma unroll
    for (int x = 0; x < VEC; ++x) tile[r * Geo<D>::LD + c0 + x] = v[x];
  }
  __device__ __forceinline__ void put_one(int r, int c, float v) const { tile[r * Geo<D>::LD + c] = v; }
};

// ---------------------------------------------------------------------------
// Dense transform of an LDS tile (fp32 FMA form)
// ---------------------------------------------------------------------------

// out[i] = sum_k tile[r_i, k] * Wl[k, c] for this thread's column c = tid % D and
// rows r_i = tid / D + i * (kBlock / D).
template <int D>
__device__ __forceinline__ void tile_times_matrix(const float* tile, const float* Wl,
                                                  float (&out)[R * D / kBlock]) {
  constexpr int RG = kBlock / D;
  constexpr int NR = R / RG;
  constexpr int LD = Geo<D>::LD;
  const int c = threadIdx.x % D;
  const int rg = threadIdx.x / D;
#pragma unroll
  for (int i = 0; i < NR; ++i) out[i] = 0.f;
  for (int k = 0; k < D; k += 4) {
    const float w0 = Wl[(k + 0) * D + c], w1 = Wl[(k + 1) * D + c];
    const float w2 = Wl[(k + 2) * D + c], w3 = Wl[(k + 3) * D + c];
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      const float4 a = *reinterpret_cast<const float4*>(tile + (rg + i * RG) * LD + k);
      out[i] = fmaf(a.x, w0, out[i]);
      out[i] = fmaf(a.y, w1, out[i]);
      out[i] = fmaf(a.z, w2, out[i]);
      out[i] = fmaf(a.w, w3, out[i]);
    }
  }
}

template <int D>
constexpr size_t fwd_lds_bytes(int vec) {
  return (static_cast<size_t>(R) * Geo<D>::LD + D * D + kBlock * vec + D) * sizeof(float) +
         (R + 4) * sizeof(int);
}
template <int D>
constexpr size_t bwd_lds_bytes(int vec) {
  return (2 * static_cast<size_t>(R) * Geo<D>::LD + D * D + kBlock * vec + D) * sizeof(float) +
         (R + 4) * sizeof(int);
}

// ---------------------------------------------------------------------------
// Forward, hidden layer: Y = relu((A_hat X) W^k)  [+ t = Y w_out^k]
// ---------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kBlock) void fwd_hidden_kernel(GraphView g, const T* __restrict__ X,
                                                            const float* __restrict__ W,
                                                            int w_stride, T* __restrict__ Y,
                                                            const float* __restrict__ w_out,
                                                            int wout_stride, float* __restrict__ t,
                                                            const float* __restrict__ heavy_partial) {
  constexpr int VEC = Store<T>::VEC;
  constexpr int LD = Geo<D>::LD;
  constexpr int RG = kBlock / D;
  constexpr int NR = R / RG;
  extern __shared__ __align__(16) unsigned char smem[];
  float* tile = reinterpret_cast<float*>(smem);
  float* Wl = tile + R * LD;
  float* red = Wl + D * D;
  float* wo = red + kBlock * VEC;
  int* hlist = reinterpret_cast<int*>(wo + D);

  const int k = g.blk_k[blockIdx.x];
  if (k < 0) return;
  const int s = g.blk_s[blockIdx.x];
  const int tid = threadIdx.x;
  const float* Wk = W + static_cast<size_t>(k) * w_stride;
  for (int idx = tid; idx < D * D; idx += kBlock) Wl[idx] = Wk[idx];
  if (w_out != nullptr && tid < D) wo[tid] = w_out[static_cast<size_t>(k) * wout_stride + tid];
  PlainSrc<T, D> src{X, g.sb};
  const int rbeg = g.part_rows[k], rend = g.part_rows[k + 1];
  const int c = tid % D, rg = tid / D;
  for (int row0 = rbeg + s * R; row0 < rend; row0 += g.blk_S[blockIdx.x] * R) {
    const int nrows = min(R, rend - row0);
    aggregate_tile<T, D>(g, src, TileSink<D>{tile}, row0, nrows, red, hlist, heavy_partial);
    __syncthreads();
    float out[NR];
    tile_times_matrix<D>(tile, Wl, out);
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      const int r = rg + i * RG;
      out[i] = Store<T>::as_stored(fmaxf(out[i], 0.f));
      if (r < nrows) Store<T>::put(Y + static_cast<size_t>(row0 + r) * D + c, out[i]);
    }
    if (w_out != nullptr) {
      __syncthreads();
#pragma unroll
      for (int i = 0; i < NR; ++i) tile[(rg + i * RG) * LD + c] = out[i];
      __syncthreads();
      if (tid < nrows) {
        float acc = 0.f;
        for (int cc = 0; cc < D; ++cc) acc = fmaf(tile[tid * LD + cc], wo[cc], acc);
        t[row0 + tid] = acc;
      }
    }
    __syncthreads();
  }
}

// t = X w^k for L = 1 (no hidden layer).
template <typename T, int D>
__global__ __launch_bounds__(kBlock) void fwd_gemv_kernel(GraphView g, const T* __restrict__ X,
                                                          const float* __restrict__ w, int w_stride,
                                                          float* __restrict__ t) {
  const int k = g.nblk_k[blockIdx.x];
  if (k < 0) return;
  const int s = g.nblk_s[blockIdx.x];
  const int rbeg = g.part_rows[k], rend = g.part_rows[k + 1];
  const float* wk = w + static_cast<size_t>(k) * w_stride;
  for (int row0 = rbeg + s * kNarrowRows; row0 < rend; row0 += g.nblk_S[blockIdx.x] * kNarrowRows) {
    const int i = row0 + threadIdx.x;
    if (i < rend) {
      float acc = 0.f;
      for (int cc = 0; cc < D; ++cc)
        acc = fmaf(Store<T>::get(X + static_cast<size_t>(i) * D + cc), wk[cc], acc);
      t[i] = acc;
    }
  }
}

// ---------------------------------------------------------------------------
// Backward of a hidden layer (see BwdArgs)
// ---------------------------------------------------------------------------
template <typename T, int D, bool LAST, bool TO_EMBED>
__global__ __launch_bounds__(kBlock) void bwd_hidden_kernel(GraphView g, BwdArgs a) {
  constexpr int VEC = Store<T>::VEC;
  constexpr int LPR = D / VEC;
  constexpr int LD = Geo<D>::LD;
  constexpr int RG = kBlock / D;
  constexpr int NR = R / RG;
  constexpr int AG = kBlock / D;                       // row groups of the D x D gradient
  constexpr int NA = (D * D >= kBlock) ? (D * D / kBlock) : 1;
  extern __shared__ __align__(16) unsigned char smem[];
  float* tile = reinterpret_cast<float*>(smem);        // G_T tile
  float* hp = tile + R * LD;                           // Hprev tile
  float* Wt = hp + R * LD;                             // Wt[b, a] = W[a, b]
  float* red = Wt + D * D;
  float* gtl = red + kBlock * VEC;                     // g_t of the tile rows (LAST)
  int* hlist = reinterpret_cast<int*>(gtl + D);

  const int k = g.blk_k[blockIdx.x];
  if (k < 0) return;
  const AdamStep ad = a.adam.for_part(k);
  const int s = g.blk_s[blockIdx.x];
  const int tid = threadIdx.x;
  const T* Hprev = static_cast<const T*>(a.Hprev);
  const float* Wk = a.W + static_cast<size_t>(k) * a.w_stride;
  for (int idx = tid; idx < D * D; idx += kBlock) Wt[(idx % D) * D + idx / D] = Wk[idx];

  PlainSrc<T, D> psrc{static_cast<const T*>(a.GZ_in), g.sb};
  LastSrc<T, D> lsrc{static_cast<const T*>(a.Hcur), g.sb, a.g_t, a.w_out, a.wout_stride, {}};
  if (LAST) lsrc.set_part(k, (tid % LPR) * VEC);

  const int rbeg = g.part_rows[k], rend = g.part_rows[k + 1];
  const int c = tid % D, rg = tid / D;
  const bool gw_active = (D * D >= kBlock) || (rg < D);
  float gw[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) gw[i] = 0.f;
  float gwo = 0.f;  // gradient of w_out[c] (LAST, threads tid < D)

  for (int row0 = rbeg + s * R; row0 < rend; row0 += g.blk_S[blockIdx.x] * R) {
    const int nrows = min(R, rend - row0);
    if (LAST)
      aggregate_tile<T, D>(g, lsrc, TileSink<D>{tile}, row0, nrows, red, hlist, a.heavy_partial);
    else
      aggregate_tile<T, D>(g, psrc, TileSink<D>{tile}, row0, nrows, red, hlist, a.heavy_partial);
    // Hprev tile -> LDS (fp32), zero beyond the tile's rows
    for (int idx = tid; idx < R * LPR; idx += kBlock) {
      const int r = idx / LPR, cc = (idx % LPR) * VEC;
      float v[VEC];
      if (r < nrows) {
        Store<T>::load(Hprev + static_cast<size_t>(row0 + r) * D + cc, v);
      } else {
#pragma unroll
        for (int x = 0; x < VEC; ++x) v[x] = 0.f;
      }
#pragma unroll
      for (int x = 0; x < VEC; ++x) hp[r * LD + cc + x] = v[x];
    }
    if (LAST && tid < D) {
      const T* Hcur = static_cast<const T*>(a.Hcur);
      for (int r = 0; r < nrows; ++r)
        gwo = fmaf(Store<T>::get(Hcur + static_cast<size_t>(row0 + r) * D + tid), a.g_t[row0 + r], gwo);
    }
    __syncthreads();
    // gW[a_, c] += sum_r Hprev[r, a_] * G_T[r, c]
    if (gw_active) {
      for (int r = 0; r < R; ++r) {
        const float gt = tile[r * LD + c];
#pragma unroll
        for (int i = 0; i < NA; ++i) gw[i] = fmaf(hp[r * LD + rg + i * AG], gt, gw[i]);
      }
    }
    // G_Hprev[r, c] = sum_b G_T[r, b] * W[c, b]
    if (!(TO_EMBED && a.mode == EMBED_SKIP)) {
      float gh[NR];
      tile_times_matrix<D>(tile, Wt, gh);
#pragma unroll
      for (int i = 0; i < NR; ++i) {
        const int r = rg + i * RG;
        if (r >= nrows) continue;
        const size_t idx = static_cast<size_t>(row0 + r) * D + c;
        if (TO_EMBED) {
          if (a.mode == EMBED_WRITE_GRAD) {
            a.gE[idx] = gh[i];
          } else {
            const float gq = gh[i];
            const float m = ad.b1 * a.mE[idx] + (1.f - ad.b1) * gq;
            const float v = ad.b2 * a.vE[idx] + (1.f - ad.b2) * gq * gq;
            const float upd = (m * ad.inv_bc1) / (sqrtf(v) * ad.inv_sqrt_bc2 + ad.eps);
            const float e = a.E[idx] - ad.lr * upd;
            a.mE[idx] = m;
            a.vE[idx] = v;
            a.E[idx] = e;
            if (sizeof(T) == 2) Store<T>::put(static_cast<T*>(a.Eb) + idx, e);
          }
        } else {
          Store<T>::put(static_cast<T*>(a.GZ_out) + idx, hp[r * LD + c] > 0.f ? gh[i] : 0.f);
        }
      }
    }
    __syncthreads();
  }
  if (gw_active) {
#pragma unroll
    for (int i = 0; i < NA; ++i)
      a.gW_partial[static_cast<size_t>(blockIdx.x) * D * D + (rg + i * AG) * D + c] = gw[i];
  }
  if (LAST && tid < D) a.gwout_partial[static_cast<size_t>(blockIdx.x) * D + tid] = gwo;
}

// L = 1: p = sigmoid(A_hat (E w)).  gw partial = sum_i X[i,:] g_t[i]; gE[i,:] = g_t[i] w.
template <typename T, int D>
__global__ __launch_bounds__(kBlock) void bwd_single_kernel(GraphView g, BwdArgs a) {
  constexpr int RG = kBlock / D;
  const int k = g.blk_k[blockIdx.x];
  if (k < 0) return;
  const AdamStep ad = a.adam.for_part(k);
  const int s = g.blk_s[blockIdx.x];
  const int tid = threadIdx.x;
  const int c = tid % D, rg = tid / D;
  __shared__ float red[kBlock];
  const T* X = static_cast<const T*>(a.Hprev);
  const float wc = a.w_out[static_cast<size_t>(k) * a.wout_stride + c];
  const int rbeg = g.part_rows[k], rend = g.part_rows[k + 1];
  float gw = 0.f;
  for (int row0 = rbeg + s * R; row0 < rend; row0 += g.blk_S[blockIdx.x] * R) {
    const int nrows = min(R, rend - row0);
    for (int r = rg; r < nrows; r += RG) {
      const size_t idx = static_cast<size_t>(row0 + r) * D + c;
      const float gt = a.g_t[row0 + r];
      gw = fmaf(Store<T>::get(X + idx), gt, gw);
      const float gq = gt * wc;
      if (a.mode == EMBED_WRITE_GRAD) {
        a.gE[idx] = gq;
      } else if (a.mode == EMBED_ADAM) {
        const float m = ad.b1 * a.mE[idx] + (1.f - ad.b1) * gq;
        const float v = ad.b2 * a.vE[idx] + (1.f - ad.b2) * gq * gq;
        const float upd = (m * ad.inv_bc1) / (sqrtf(v) * ad.inv_sqrt_bc2 + ad.eps);
        const float e = a.E[idx] - ad.lr * upd;
        a.mE[idx] = m;
        a.vE[idx] = v;
        a.E[idx] = e;
        if (sizeof(T) == 2) Store<T>::put(static_cast<T*>(a.Eb) + idx, e);
      }
    }
  }
  red[tid] = gw;
  __syncthreads();
  if (tid < D) {
    float sacc = 0.f;
    for (int q = 0; q < RG; ++q) sacc += red[q * D + tid];
    a.gwout_partial[static_cast<size_t>(blockIdx.x) * D + tid] = sacc;
  }
}

// ---------------------------------------------------------------------------
// Width-1 passes: y_i = f_self(i) + sum_{j in N(i)} f(j), then an epilogue per row
// ---------------------------------------------------------------------------

// Loss of subgraph k from the workgroup partials of one epoch: the lanes of a wavefront add
// the partials of k in a strided, fixed order, then a butterfly forms the total (every lane
// returns it).
__device__ inline double subgraph_loss(const GraphView& g, const double* __restrict__ partial, int k,
                                       int lane) {
  double acc = 0.0;
  for (int q = g.loss_ptr[k] + lane; q < g.loss_ptr[k + 1]; q += 64) acc += partial[g.loss_list[q]];
  return wave_sum(acc);
}

// Sum of part_s[0..P) in a fixed order (per-thread strided sums, then thread 0 adds them);
// valid in thread 0.  Contains workgroup barriers.
__device__ inline double total_loss(const double* part_s, int P, double* tot) {
  __syncthreads();
  double mine = 0.0;
  for (int k = threadIdx.x; k < P; k += kBlock) mine += part_s[k];
  tot[threadIdx.x] = mine;
  __syncthreads();
  double acc = 0.0;
  if (threadIdx.x == 0)
    for (int q = 0; q < kBlock; ++q) acc += tot[q];
  return acc;
}

// One workgroup per set of partials (one set per epoch).  Each wavefront takes subgraphs
// k = wave, wave + 4, ...  loss_part (per-subgraph values, [sets, P]) may be null.
__global__ __launch_bounds__(kBlock) void loss_reduce_kernel(GraphView g, const double* __restrict__ partial,
                                                             int64_t set_stride,
                                                             double* __restrict__ loss_part,
                                                             double* __restrict__ loss_out) {
  extern __shared__ double part_s[];  // [P]
  __shared__ double tot[kBlock];
  partial += static_cast<int64_t>(blockIdx.x) * set_stride;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  for (int k = wave; k < g.P; k += kBlock / 64) {
    const double acc = subgraph_loss(g, partial, k, lane);
    if (lane == 0) {
      part_s[k] = acc;
      if (loss_part != nullptr) loss_part[static_cast<int64_t>(blockIdx.x) * g.P + k] = acc;
    }
  }
  const double total = total_loss(part_s, g.P, tot);
  if (threadIdx.x == 0) loss_out[blockIdx.x] = total;
}

// ---------------------------------------------------------------------------
// Best-by-loss snapshot (Alg. 1 stage 1: the best network of every subgraph is kept)
// ---------------------------------------------------------------------------

// One workgroup.  The losses of this epoch, summed exactly as loss_reduce_kernel sums them,
// are compared with the lowest seen so far, per model: a subgraph (models == P) or the
// whole batch (models == 1).  A subgraph without loss partials is not being trained and is
// not offered.  improved[u] tells the copy kernel which models to store.
__global__ __launch_bounds__(kBlock) void best_update_kernel(GraphView g, const double* __restrict__ partial,
                                                             int models, double* __restrict__ best_loss,
                                                             int* __restrict__ improved,
                                                             int* __restrict__ has_best) {
  extern __shared__ double part_s[];  // [P]
  __shared__ double tot[kBlock];
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  for (int k = wave; k < g.P; k += kBlock / 64) {
    const double acc = subgraph_loss(g, partial, k, lane);
    if (lane == 0) {
      part_s[k] = acc;
      if (models != 1) {
        const bool better = g.loss_ptr[k + 1] > g.loss_ptr[k] && acc < best_loss[k];
        improved[k] = better ? 1 : 0;
        if (better) {
          best_loss[k] = acc;
          has_best[k] = 1;
        }
      }
    }
  }
  const double total = total_loss(part_s, g.P, tot);
  if (models == 1 && threadIdx.x == 0) {
    const bool better = g.loss_ptr[g.P] > g.loss_ptr[0] && total < best_loss[0];
    improved[0] = better ? 1 : 0;
    if (better) {
      best_loss[0] = total;
      has_best[0] = 1;
    }
  }
}

struct ParamCopy {
  const float* E_src = nullptr;
  float* E_dst = nullptr;
  const float* W_src[3] = {};
  float* W_dst[3] = {};
  int w_elems[3] = {};  // per weight set
  int num_w = 0;
};

// Copies the parameters of the models with flag[u] != 0.  blockIdx.x < P: the embedding
// rows of subgraph x (row width D floats, D % 4 == 0); blockIdx.x = P + l: weight tensor l
// of every flagged model.  The gridDim.y workgroups of one x share the work in a strided
// loop, four 16-byte accesses in flight per lane; the embedding is read and written past
// the caches.
__global__ __launch_bounds__(kBlock) void param_copy_kernel(GraphView g, int models, int D,
                                                            const int* __restrict__ flag, ParamCopy c) {
  const int y = blockIdx.x;
  const int64_t stride = static_cast<int64_t>(gridDim.y) * kBlock;
  const int64_t first = static_cast<int64_t>(blockIdx.y) * kBlock + threadIdx.x;
  if (y < g.P) {
    if (!flag[models == 1 ? 0 : y]) return;
    const int64_t i0 = static_cast<int64_t>(g.part_rows[y]) * (D / 4);
    const int64_t i1 = static_cast<int64_t>(g.part_rows[y + 1]) * (D / 4);
    for (int64_t i = i0 + first; i < i1; i += 4 * stride) {
      typedef float f32x4_t __attribute__((ext_vector_type(4)));
      const f32x4_t* src = reinterpret_cast<const f32x4_t*>(c.E_src);
      f32x4_t* dst = reinterpret_cast<f32x4_t*>(c.E_dst);
      f32x4_t v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (i + u * stride < i1) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (i + u * stride < i1) __builtin_nontemporal_store(v[u], dst + i + u * stride);
    }
  } else {
    const int l = y - g.P;
    if (l >= c.num_w) return;
    const int elems = c.w_elems[l];
    for (int u = 0; u < models; ++u) {
      if (!flag[u]) continue;
      const int64_t base = static_cast<int64_t>(u) * elems;
      for (int64_t e = first; e < elems; e += stride) c.W_dst[l][base + e] = c.W_src[l][base + e];
    }
  }
}

// ---------------------------------------------------------------------------
// Adam on the weight matrices (with the fixed-order reduction of the partials)
// ---------------------------------------------------------------------------
struct WeightTensors {
  WeightTensor t[3];
  int count = 0;
};

// Which tensor, weight set and element a global element index stands for.
struct WeightElem {
  int which, k, idx;
  int64_t gid;  // index inside the tensor
};
__device__ inline WeightElem locate_weight(int Pw, const WeightTensors& wts, int64_t gid) {
  int which = 0;
  while (which < wts.count && gid >= static_cast<int64_t>(Pw) * wts.t[which].elems) {
    gid -= static_cast<int64_t>(Pw) * wts.t[which].elems;
    ++which;
  }
  WeightElem e{which, 0, 0, gid};
  if (which < wts.count) {
    e.k = static_cast<int>(gid / wts.t[which].elems);
    e.idx = static_cast<int>(gid % wts.t[which].elems);
  }
  return e;
}

// Sum of 16 partials of one element, pairwise: 16 loads in flight.
__device__ inline float sum16(const float* base, const int* __restrict__ list, int elems) {
  float v[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) v[u] = base[static_cast<size_t>(list[u]) * elems];
#pragma unroll
  for (int w = 1; w < 16; w *= 2)
#pragma unroll
    for (int u = 0; u < 16; u += 2 * w) v[u] += v[u + w];
  return v[0];
}

__device__ inline void adam_on_weight(const WeightTensor& wt, int64_t gid, float gsum, const AdamStep& adk,
                                      int update) {
  if (wt.grad_out != nullptr) wt.grad_out[gid] = gsum;
  if (update) {
    const float m = adk.b1 * wt.m[gid] + (1.f - adk.b1) * gsum;
    const float v = adk.b2 * wt.v[gid] + (1.f - adk.b2) * gsum * gsum;
    wt.m[gid] = m;
    wt.v[gid] = v;
    wt.W[gid] -= adk.lr * (m * adk.inv_bc1) / (sqrtf(v) * adk.inv_sqrt_bc2 + adk.eps);
  }
}

// One thread per weight of every tensor.  The partials are added in groups of 16
// (pairwise inside a group, groups in list order) so that 16 loads are in flight.
// DC > 0 (the feature width): the workgroups from weight_blocks on pre-reduce, for the next
// forward pass, the chunks of the rows with very many neighbours from the bf16 working copy
// of the embeddings, which the launch before this one has finished writing.
template <int DC>
__global__ __launch_bounds__(kBlock) void adam_w_kernel(int Pw, WeightTensors wts, AdamStep ad, int update,
                                                        int weight_blocks, GraphView g,
                                                        const bf16_t* __restrict__ Eb,
                                                        float* __restrict__ chunk_partial) {
  if constexpr (DC > 0) {
    __shared__ float red[kBlock * 8];
    if (static_cast<int>(blockIdx.x) >= weight_blocks) {
      const int ch = blockIdx.x - weight_blocks;
      if (g.chunk_part[ch] < 0) return;  // the row's subgraph sits out
      reduce_chunk<DC>(g, ChunkPlainRows<DC>{Eb}, chunk_partial, ch, red);
      return;
    }
  }
  const WeightElem e = locate_weight(Pw, wts, static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x);
  if (e.which >= wts.count) return;
  const WeightTensor& wt = wts.t[e.which];
  const float* base = wt.partial + e.idx;
  float gsum = 0.f;
  int q = wt.blk_ptr[e.k];
  const int q1 = wt.blk_ptr[e.k + 1];
  if (q == q1) {  // no workgroup produced a gradient for this weight set: it sits out
    if (wt.grad_out != nullptr) wt.grad_out[e.gid] = 0.f;
    return;
  }
  for (; q + 16 <= q1; q += 16) gsum += sum16(base, wt.blk_list + q, wt.elems);
  for (; q < q1; ++q) gsum += base[static_cast<size_t>(wt.blk_list[q]) * wt.elems];
  adam_on_weight(wt, e.gid, gsum, ad.for_part(e.k), update);
}

// The same for few weight sets with very many partials each (one subgraph holding the whole
// graph): a workgroup of S wavefronts serves 64 weights; wavefront w adds the groups of 16
// partials number w, w + S, ...; the S sums are then added in order, the leftover partials
// (fewer than 16) last.
constexpr int kAdamSplit = 16;
__global__ __launch_bounds__(64 * kAdamSplit) void adam_w_split_kernel(int Pw, WeightTensors wts, AdamStep ad,
                                                                       int update) {
  __shared__ float red[kAdamSplit][64];
  const int lane = threadIdx.x % 64, w = threadIdx.x / 64;
  const WeightElem e = locate_weight(Pw, wts, static_cast<int64_t>(blockIdx.x) * 64 + lane);
  const bool live = e.which < wts.count;
  const WeightTensor& wt = wts.t[live ? e.which : 0];
  int q0 = 0, q1 = 0;
  if (live) {
    q0 = wt.blk_ptr[e.k];
    q1 = wt.blk_ptr[e.k + 1];
  }
  const float* base = wt.partial + e.idx;
  const int groups = (q1 - q0) / 16;
  float mine = 0.f;
  for (int gq = w; gq < groups; gq += kAdamSplit) mine += sum16(base, wt.blk_list + q0 + gq * 16, wt.elems);
  red[w][lane] = mine;
  __syncthreads();
  if (w != 0 || !live) return;
  if (q0 == q1) {
    if (wt.grad_out != nullptr) wt.grad_out[e.gid] = 0.f;
    return;
  }
  float gsum = 0.f;
  for (int u = 0; u < kAdamSplit; ++u) gsum += red[u][lane];
  for (int q = q0 + groups * 16; q < q1; ++q) gsum += base[static_cast<size_t>(wt.blk_list[q]) * wt.elems];
  adam_on_weight(wt, e.gid, gsum, ad.for_part(e.k), update);
}

// Sec. 3.2, input processing: X[i, :] = softmax((X[i, :] + g[i, :]) / tau) in place, with
// g = -log(-log(U[i, :])).  One thread per row (runs once per parameter upload).
__global__ __launch_bounds__(kBlock) void gumbel_softmax_rows_kernel(int n, int D, float* __restrict__ X,
                                                                     const float* __restrict__ U, float inv_tau) {
  const int i = blockIdx.x * kBlock + threadIdx.x;
  if (i >= n) return;
  float* x = X + static_cast<size_t>(i) * D;
  const float* u = U + static_cast<size_t>(i) * D;
  float top = -INFINITY;
  for (int c = 0; c < D; ++c) {
    const float y = (x[c] - logf(-logf(u[c]))) * inv_tau;
    x[c] = y;
    top = fmaxf(top, y);
  }
  float sum = 0.f;
  for (int c = 0; c < D; ++c) {
    const float w = expf(x[c] - top);
    x[c] = w;
    sum += w;
  }
  const float inv = 1.f / sum;
  for (int c = 0; c < D; ++c) x[c] *= inv;
}

__global__ __launch_bounds__(kBlock) void to_bf16_kernel(const float* __restrict__ src,
                                                         bf16_t* __restrict__ dst, int64_t count) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (i < count) dst[i] = f32_to_bf16(src[i]);
}

__global__ __launch_bounds__(kBlock) void from_bf16_kernel(const bf16_t* __restrict__ src,
                                                           float* __restrict__ dst, int64_t count) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (i < count) dst[i] = bf16_to_f32(src[i]);
}

template <typename K>
void allow_lds(K kernel, size_t bytes) {
  if (bytes > 48 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
}

}  // namespace

// ---------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------
#define GCO_DISPATCH_D(T, D, ...)                                   \
  switch (D) {                                                      \
    case 8: if (sizeof(T) == 4) { constexpr int DD = 8; __VA_ARGS__; } break;   \
    case 16: if (sizeof(T) == 4) { constexpr int DD = 16; __VA_ARGS__; } break; \
    case 32: { constexpr int DD = 32; __VA_ARGS__; } break;         \
    case 64: { constexpr int DD = 64; __VA_ARGS__; } break;         \
    case 128: { constexpr int DD = 128; __VA_ARGS__; } break;       \
    default: break;                                                 \
  }

template <typename T, int D>
static void fwd_hidden_t(const Launch& ln, const GraphView& g, const void* X, const float* W,
                         int w_stride, void* Y, const float* w_out, int wout_stride, float* t,
                         float* heavy_partial) {
  if (g.num_chunks > 0) {
    ln.begin(KK_HEAVY);
    PlainSrc<T, D> src{static_cast<const T*>(X), g.sb};
    heavy_wide_kernel<T, D, PlainSrc<T, D>><<<g.num_chunks, kBlock, 0, ln.st>>>(g, src, heavy_partial);
    ln.end(KK_HEAVY);
  }
  const size_t lds = fwd_lds_bytes<D>(Store<T>::VEC);
  allow_lds(fwd_hidden_kernel<T, D>, lds);
  ln.begin(KK_FWD_HIDDEN);
  fwd_hidden_kernel<T, D><<<g.num_blocks, kBlock, lds, ln.st>>>(
      g, static_cast<const T*>(X), W, w_stride, static_cast<T*>(Y), w_out, wout_stride, t, heavy_partial);
  ln.end(KK_FWD_HIDDEN);
}

void launch_fwd_hidden(const Launch& ln, int storage, int D, const GraphView& g, const void* X,
                       const float* W, int w_stride, void* Y, const float* w_out, int wout_stride,
                       float* t, float* heavy_partial, bool partial_ready) {
  if (storage == GCO_STORAGE_BF16) {
    launch_fwd_hidden_bf16(ln, D, g, X, W, w_stride, Y, w_out, wout_stride, t, heavy_partial, partial_ready);
  } else {
    GCO_DISPATCH_D(float, D, (fwd_hidden_t<float, DD>(ln, g, X, W, w_stride, Y, w_out, wout_stride, t, heavy_partial)))
  }
}

void launch_fwd_gemv(const Launch& ln, int storage, int D, const GraphView& g, const void* X,
                     const float* w, int w_stride, float* t) {
  ln.begin(KK_FWD_GEMV);
  if (storage == GCO_STORAGE_BF16) {
    GCO_DISPATCH_D(bf16_t, D, (fwd_gemv_kernel<bf16_t, DD><<<g.num_nblocks, kBlock, 0, ln.st>>>(g, static_cast<const bf16_t*>(X), w, w_stride, t)))
  } else {
    GCO_DISPATCH_D(float, D, (fwd_gemv_kernel<float, DD><<<g.num_nblocks, kBlock, 0, ln.st>>>(g, static_cast<const float*>(X), w, w_stride, t)))
  }
  ln.end(KK_FWD_GEMV);
}

void launch_best_update(const Launch& ln, const GraphView& g, const double* loss_partial, int models,
                        double* best_loss, int* improved, int* has_best) {
  const size_t lds = static_cast<size_t>(g.P) * sizeof(double);
  allow_lds(best_update_kernel, lds);
  ln.begin(KK_BEST);
  best_update_kernel<<<1, kBlock, lds, ln.st>>>(g, loss_partial, models, best_loss, improved, has_best);
  ln.end(KK_BEST);
}

void launch_param_copy(const Launch& ln, const GraphView& g, int models, int D, const int* flag,
                       const float* E_src, float* E_dst, const float* const* W_src, float* const* W_dst,
                       const int* w_elems, int num_w) {
  ParamCopy c;
  c.E_src = E_src;
  c.E_dst = E_dst;
  c.num_w = num_w;
  for (int l = 0; l < num_w; ++l) {
    c.W_src[l] = W_src[l];
    c.W_dst[l] = W_dst[l];
    c.w_elems[l] = w_elems[l];
  }
  const int per_part = std::max(1, (kWideBlocks + g.P - 1) / g.P);
  ln.begin(KK_BEST);
  param_copy_kernel<<<dim3(g.P + num_w, per_part), kBlock, 0, ln.st>>>(g, models, D, flag, c);
  ln.end(KK_BEST);
}

void launch_loss_reduce(const Launch& ln, const GraphView& g, const double* loss_partial, int sets,
                        int64_t set_stride, double* loss_part, double* loss_out) {
  if (sets <= 0) return;
  const size_t lds = static_cast<size_t>(g.P) * sizeof(double);
  allow_lds(loss_reduce_kernel, lds);
  ln.begin(KK_LOSS_REDUCE);
  loss_reduce_kernel<<<sets, kBlock, lds, ln.st>>>(g, loss_partial, set_stride, loss_part, loss_out);
  ln.end(KK_LOSS_REDUCE);
}

template <typename T, int D>
static void bwd_hidden_t(const Launch& ln, bool last, bool to_embed, const GraphView& g,
                         const BwdArgs& a) {
  const GraphView gt = transposed(g);
  if (g.num_chunks > 0) {
    ln.begin(KK_HEAVY);
    if (last) {
      LastSrc<T, D> src{static_cast<const T*>(a.Hcur), gt.sb, a.g_t, a.w_out, a.wout_stride, {}};
      heavy_wide_kernel<T, D, LastSrc<T, D>><<<g.num_chunks, kBlock, 0, ln.st>>>(gt, src, a.heavy_partial);
    } else {
      PlainSrc<T, D> src{static_cast<const T*>(a.GZ_in), gt.sb};
      heavy_wide_kernel<T, D, PlainSrc<T, D>><<<g.num_chunks, kBlock, 0, ln.st>>>(gt, src, a.heavy_partial);
    }
    ln.end(KK_HEAVY);
  }
  const size_t lds = bwd_lds_bytes<D>(Store<T>::VEC);
  const int kind = to_embed ? KK_BWD_EMBED : KK_BWD_HIDDEN;
  ln.begin(kind);
#define GCO_BWD(L_, E_)                                                        \
  {                                                                            \
    allow_lds(bwd_hidden_kernel<T, D, L_, E_>, lds);                           \
    bwd_hidden_kernel<T, D, L_, E_><<<g.num_blocks, kBlock, lds, ln.st>>>(gt, a); \
  }
  if (last && to_embed) GCO_BWD(true, true)
  else if (last) GCO_BWD(true, false)
  else if (to_embed) GCO_BWD(false, true)
  else GCO_BWD(false, false)
#undef GCO_BWD
  ln.end(kind);
}

void launch_bwd_hidden(const Launch& ln, int storage, int D, bool last, bool to_embed,
                       const GraphView& g, const BwdArgs& a) {
  if (storage == GCO_STORAGE_BF16) {
    launch_bwd_hidden_bf16(ln, D, last, to_embed, transposed(g), a);
  } else {
    GCO_DISPATCH_D(float, D, (bwd_hidden_t<float, DD>(ln, last, to_embed, g, a)))
  }
}

void launch_bwd_single(const Launch& ln, int storage, int D, const GraphView& g, const BwdArgs& a) {
  ln.begin(KK_BWD_EMBED);
  if (storage == GCO_STORAGE_BF16) {
    GCO_DISPATCH_D(bf16_t, D, (bwd_single_kernel<bf16_t, DD><<<g.num_blocks, kBlock, 0, ln.st>>>(g, a)))
  } else {
    GCO_DISPATCH_D(float, D, (bwd_single_kernel<float, DD><<<g.num_blocks, kBlock, 0, ln.st>>>(g, a)))
  }
  ln.end(KK_BWD_EMBED);
}

void launch_adam_w(const Launch& ln, int Pw, const WeightTensor* tensors, int count, const AdamStep& adam,
                   bool update, bool many_partials, const ChunkTail* tail) {
  WeightTensors wts;
  wts.count = count;
  int64_t total = 0;
  for (int i = 0; i < count; ++i) {
    wts.t[i] = tensors[i];
    total += static_cast<int64_t>(Pw) * tensors[i].elems;
  }
  ln.begin(KK_ADAM_W);
  if (many_partials) {
    const int blocks = static_cast<int>((total + 63) / 64);
    adam_w_split_kernel<<<blocks, 64 * kAdamSplit, 0, ln.st>>>(Pw, wts, adam, update ? 1 : 0);
  } else {
    const int blocks = static_cast<int>((total + kBlock - 1) / kBlock);
    const bf16_t* Eb = tail ? static_cast<const bf16_t*>(tail->X) : nullptr;
    if (tail != nullptr && tail->D == 64)
      adam_w_kernel<64><<<blocks + tail->g.num_chunks, kBlock, 0, ln.st>>>(Pw, wts, adam, update ? 1 : 0, blocks,
                                                                          tail->g, Eb, tail->partial);
    else if (tail != nullptr && tail->D == 128)
      adam_w_kernel<128><<<blocks + tail->g.num_chunks, kBlock, 0, ln.st>>>(Pw, wts, adam, update ? 1 : 0, blocks,
                                                                           tail->g, Eb, tail->partial);
    else
      adam_w_kernel<0><<<blocks, kBlock, 0, ln.st>>>(Pw, wts, adam, update ? 1 : 0, blocks, GraphView{}, nullptr,
                                                     nullptr);
  }
  ln.end(KK_ADAM_W);
}

void launch_gumbel_softmax_rows(const Launch& ln, int n, int D, float* X, const float* U, float tau) {
  const int blocks = (n + kBlock - 1) / kBlock;
  if (blocks > 0) gumbel_softmax_rows_kernel<<<blocks, kBlock, 0, ln.st>>>(n, D, X, U, 1.f / tau);
}

void launch_to_bf16(const Launch& ln, const float* src, void* dst, int64_t count) {
  const int blocks = static_cast<int>((count + kBlock - 1) / kBlock);
  if (blocks > 0)
    to_bf16_kernel<<<blocks, kBlock, 0, ln.st>>>(src, static_cast<bf16_t*>(dst), count);
}

void launch_from_bf16(const Launch& ln, const void* src, float* dst, int64_t count) {
  const int blocks = static_cast<int>((count + kBlock - 1) / kBlock);
  if (blocks > 0)
    from_bf16_kernel<<<blocks, kBlock, 0, ln.st>>>(static_cast<const bf16_t*>(src), dst, count);
}

}  // namespace gco
