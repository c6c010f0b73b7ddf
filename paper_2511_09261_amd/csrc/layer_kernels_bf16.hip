// bf16-storage versions of the fused layer kernels: the gather is as in the fp32
// kernels (fp32 accumulation), the dense transforms run on the matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
// Operand layout of that instruction, per 64-lane wavefront (lane l):
//   A (32 x 16): row l % 32, columns 8 * (l / 32) .. + 7   (8 bf16 = 16 bytes)
//   B (16 x 32): rows 8 * (l / 32) .. + 7, column l % 32
//   C (32 x 32): register r in 0..15 holds row (r / 4) * 8 + (l / 32) * 4 + r % 4,
//                column l % 32
// so both operands want their 8 values contiguous along the contracted index.
// LDS tiles are therefore kept as [row][feature] for products contracted over
// features (the layer transform, and the product with W^T in the backward pass)
// and as [feature][row] for the weight gradient, which is contracted over rows.
// Row pitches are padded by 16 bytes, which spreads 16 consecutive rows over all
// 64 LDS banks for 16-byte reads.
#include "device_utils.h"
#include "gather.h"
#include "gco_internal.h"

namespace gco {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int R = kTileRows;
static_assert(R == 64, "the wave-to-tile maps below assume 64-row tiles");

template <int D>
struct MG {
  static constexpr int PA = D + 8;                      // pitch of [row][feature] tiles (bf16)
  static constexpr int PT = R + 8;                      // pitch of [feature][row] tiles (bf16)
  static constexpr int NT = D / 32;                     // 32-wide column tiles
  static constexpr int MT = R / 32;                     // 32-high row tiles
  static constexpr int KS = D / 16;                     // k-steps of a product contracted over features
  static constexpr int WPC = (4 / NT) > 0 ? 4 / NT : 1; // waves sharing one column tile
  static constexpr int NTM = (MT + WPC - 1) / WPC;      // row tiles per wave
  static constexpr int NGW = (NT * NT + 3) / 4;         // weight-gradient tiles per wave
  static constexpr int LPR = D / 8;                     // lanes per feature row (16 bytes each)
  static constexpr int PO = D + 4;                      // pitch of the fp32 staging tile
  static constexpr size_t at_bytes = static_cast<size_t>(R) * PA * 2;
  static constexpr size_t tt_bytes = static_cast<size_t>(D) * PT * 2;
  static_assert(at_bytes % 16 == 0 && tt_bytes % 16 == 0, "tile alignment");
  static_assert(at_bytes + tt_bytes >= static_cast<size_t>(R) * PO * 4, "fp32 staging must fit");
};

__device__ __forceinline__ bf16x8 as_frag(const uint4& u) {
  bf16x8 v;
  __builtin_memcpy(&v, &u, 16);
  return v;
}

__device__ __forceinline__ uint4 pack8(const float (&v)[8]) {
  uint4 x;
  x.x = static_cast<uint32_t>(f32_to_bf16(v[0])) | (static_cast<uint32_t>(f32_to_bf16(v[1])) << 16);
  x.y = static_cast<uint32_t>(f32_to_bf16(v[2])) | (static_cast<uint32_t>(f32_to_bf16(v[3])) << 16);
  x.z = static_cast<uint32_t>(f32_to_bf16(v[4])) | (static_cast<uint32_t>(f32_to_bf16(v[5])) << 16);
  x.w = static_cast<uint32_t>(f32_to_bf16(v[6])) | (static_cast<uint32_t>(f32_to_bf16(v[7])) << 16);
  return x;
}

// Gathered rows -> bf16 LDS tiles: [row][feature] and, if asked, [feature][row].
template <int D, bool TRANSPOSED>
struct BfSink {
  bf16_t* at;
  bf16_t* tt;
  template <int VEC>
  __device__ __forceinline__ void put_vec(int r, int c0, const float (&v)[VEC]) const {
    static_assert(VEC == 8, "bf16 rows are handled 8 elements per lane");
    const uint4 x = pack8(v);
    *reinterpret_cast<uint4*>(at + r * MG<D>::PA + c0) = x;
    if (TRANSPOSED) {
      const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        tt[(c0 + 2 * q) * MG<D>::PT + r] = static_cast<bf16_t>(w[q] & 0xffffu);
        tt[(c0 + 2 * q + 1) * MG<D>::PT + r] = static_cast<bf16_t>(w[q] >> 16);
      }
    }
  }
  __device__ __forceinline__ void put_one(int r, int c, float v) const {
    const bf16_t h = f32_to_bf16(v);
    at[r * MG<D>::PA + c] = h;
    if (TRANSPOSED) tt[c * MG<D>::PT + r] = h;
  }
};

// acc[q] = (rows of row tile tm) x (this wave's column tile), contracted over the D features.
template <int D>
__device__ __forceinline__ void tile_product(const bf16_t* at, const bf16x8 (&bfrag)[MG<D>::KS],
                                             int tm0, floatx16 (&acc)[MG<D>::NTM]) {
  using M = MG<D>;
  const int lane = threadIdx.x % 64;
#pragma unroll
  for (int q = 0; q < M::NTM; ++q) {
    const int tm = tm0 + q * M::WPC;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[q][r] = 0.f;
    if (tm < M::MT) {
      const bf16_t* arow = at + (tm * 32 + lane % 32) * M::PA + 8 * (lane / 32);
#pragma unroll
      for (int ks = 0; ks < M::KS; ++ks) {
        const bf16x8 af = as_frag(*reinterpret_cast<const uint4*>(arow + ks * 16));
        acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfrag[ks], acc[q], 0, 0, 0);
      }
    }
  }
}

template <int D>
constexpr size_t fwd_lds() {
  return MG<D>::at_bytes + kBlock * 8 * sizeof(float) + D * sizeof(float) + (R + 4) * sizeof(int);
}
template <int D>
constexpr size_t bwd_lds() {
  return MG<D>::at_bytes + 2 * MG<D>::tt_bytes + kBlock * 8 * sizeof(float) + (R + 4) * sizeof(int);
}

// ---------------------------------------------------------------------------
// Forward: Y = relu((A_hat X) W^k)  [+ t = Y w_out^k]
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kBlock) void fwd_hidden_bf16_kernel(
    GraphView g, const bf16_t* __restrict__ X, const float* __restrict__ W, int w_stride,
    bf16_t* __restrict__ Y, const float* __restrict__ w_out, int wout_stride, float* __restrict__ t,
    const float* __restrict__ heavy_partial) {
  using M = MG<D>;
  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* at = reinterpret_cast<bf16_t*>(smem);
  float* red = reinterpret_cast<float*>(smem + M::at_bytes);
  float* wo = red + kBlock * 8;
  int* hlist = reinterpret_cast<int*>(wo + D);

  const int k = g.blk_k[blockIdx.x];
  if (k < 0) return;
  const int s = g.blk_s[blockIdx.x];
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int tn = wave % M::NT, tm0 = wave / M::NT;
  const float* Wk = W + static_cast<size_t>(k) * w_stride;
  // B operand: B[kk][j] = W[kk][j], j = tn * 32 + lane % 32, kept in registers
  bf16x8 bfrag[M::KS];
#pragma unroll
  for (int ks = 0; ks < M::KS; ++ks) {
    float v[8];
#pragma unroll
    for (int x = 0; x < 8; ++x) v[x] = Wk[(ks * 16 + 8 * (lane / 32) + x) * D + tn * 32 + lane % 32];
    bfrag[ks] = as_frag(pack8(v));
  }
  if (w_out != nullptr && tid < D) wo[tid] = w_out[static_cast<size_t>(k) * wout_stride + tid];
  PlainSrc<bf16_t, D> src{X, g.sb};
  const BfSink<D, false> sink{at, nullptr};
  const int rbeg = g.part_rows[k], rend = g.part_rows[k + 1];
  for (int row0 = rbeg + s * R; row0 < rend; row0 += g.S * R) {
    const int nrows = min(R, rend - row0);
    aggregate_tile<bf16_t, D>(g, src, sink, row0, nrows, red, hlist, heavy_partial);
    floatx16 acc[M::NTM];
    tile_product<D>(at, bfrag, tm0, acc);
    __syncthreads();  // every wave has read its A fragments: the tile can be reused for Y
#pragma unroll
    for (int q = 0; q < M::NTM; ++q) {
      const int tm = tm0 + q * M::WPC;
      if (tm < M::MT) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = tm * 32 + (r / 4) * 8 + (lane / 32) * 4 + r % 4;
          at[i * M::PA + tn * 32 + lane % 32] = f32_to_bf16(fmaxf(acc[q][r], 0.f));
        }
      }
    }
    __syncthreads();
    for (int idx = tid; idx < R * M::LPR; idx += kBlock) {
      const int r = idx / M::LPR, c0 = (idx % M::LPR) * 8;
      if (r < nrows)
        *reinterpret_cast<uint4*>(Y + static_cast<size_t>(row0 + r) * D + c0) =
            *reinterpret_cast<const uint4*>(at + r * M::PA + c0);
    }
    if (w_out != nullptr) {  // t[r] = sum_c Y[r, c] * w_out[c]: four lanes per row
      const int r = tid / 4, qd = tid % 4;
      float part = 0.f;
      for (int c = qd * (D / 4); c < (qd + 1) * (D / 4); ++c)
        part = fmaf(bf16_to_f32(at[r * M::PA + c]), wo[c], part);
      part += __shfl_xor(part, 1, 64);
      part += __shfl_xor(part, 2, 64);
      if (qd == 0 && r < nrows) t[row0 + r] = part;
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------
// Backward of a hidden layer (see BwdArgs in gco_internal.h)
// ---------------------------------------------------------------------------
template <int D, bool LAST, bool TO_EMBED>
__global__ __launch_bounds__(kBlock) void bwd_hidden_bf16_kernel(GraphView g, BwdArgs a) {
  using M = MG<D>;
  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* at = reinterpret_cast<bf16_t*>(smem);                              // G_T [row][feature]
  bf16_t* gtt = reinterpret_cast<bf16_t*>(smem + M::at_bytes);               // G_T [feature][row]
  bf16_t* hpt = reinterpret_cast<bf16_t*>(smem + M::at_bytes + M::tt_bytes); // Hprev [feature][row]
  float* red = reinterpret_cast<float*>(smem + M::at_bytes + 2 * M::tt_bytes);
  int* hlist = reinterpret_cast<int*>(red + kBlock * 8);
  float* stage = reinterpret_cast<float*>(smem);  // fp32 [R][PO], over at + gtt, after the products

  const int k = g.blk_k[blockIdx.x];
  if (k < 0) return;
  const int s = g.blk_s[blockIdx.x];
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int tn = wave % M::NT, tm0 = wave / M::NT;
  const bf16_t* Hprev = static_cast<const bf16_t*>(a.Hprev);
  const bf16_t* Hcur = static_cast<const bf16_t*>(a.Hcur);
  const float* Wk = a.W + static_cast<size_t>(k) * a.w_stride;
  const bool need_gh = !(TO_EMBED && a.mode == EMBED_SKIP);
  // B operand of G_H = G_T W^T: B[b][j] = W[j][b], j = tn * 32 + lane % 32
  bf16x8 wfrag[M::KS];
#pragma unroll
  for (int ks = 0; ks < M::KS; ++ks) {
    float v[8];
    const float4* wp = reinterpret_cast<const float4*>(
        Wk + static_cast<size_t>(tn * 32 + lane % 32) * D + ks * 16 + 8 * (lane / 32));
    const float4 w0 = wp[0], w1 = wp[1];
    v[0] = w0.x; v[1] = w0.y; v[2] = w0.z; v[3] = w0.w;
    v[4] = w1.x; v[5] = w1.y; v[6] = w1.z; v[7] = w1.w;
    wfrag[ks] = as_frag(pack8(v));
  }
  PlainSrc<bf16_t, D> psrc{static_cast<const bf16_t*>(a.GZ_in), g.sb};
  LastSrc<bf16_t, D> lsrc{Hcur, g.sb, a.g_t, a.w_out, a.wout_stride, {}};
  const int c0 = (tid % M::LPR) * 8;  // this thread's feature slice in row-chunk loops
  if (LAST) lsrc.set_part(k, c0);
  const BfSink<D, true> sink{at, gtt};

  floatx16 gw[M::NGW];
#pragma unroll
  for (int q = 0; q < M::NGW; ++q)
#pragma unroll
    for (int r = 0; r < 16; ++r) gw[q][r] = 0.f;
  float gwo[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  const int rbeg = g.part_rows[k], rend = g.part_rows[k + 1];
  for (int row0 = rbeg + s * R; row0 < rend; row0 += g.S * R) {
    const int nrows = min(R, rend - row0);
    if (LAST)
      aggregate_tile<bf16_t, D>(g, lsrc, sink, row0, nrows, red, hlist, a.heavy_partial);
    else
      aggregate_tile<bf16_t, D>(g, psrc, sink, row0, nrows, red, hlist, a.heavy_partial);
    // Hprev tile, transposed into LDS (zero beyond the tile's rows)
    for (int idx = tid; idx < R * M::LPR; idx += kBlock) {
      const int r = idx / M::LPR;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (r < nrows) v = *reinterpret_cast<const uint4*>(Hprev + static_cast<size_t>(row0 + r) * D + c0);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        hpt[(c0 + 2 * q) * M::PT + r] = static_cast<bf16_t>(w[q] & 0xffffu);
        hpt[(c0 + 2 * q + 1) * M::PT + r] = static_cast<bf16_t>(w[q] >> 16);
      }
      if (LAST && r < nrows) {  // gradient of w_out: sum_r Hcur[r, c] * g_t[r]
        float h[8];
        Store<bf16_t>::load(Hcur + static_cast<size_t>(row0 + r) * D + c0, h);
        const float gt = a.g_t[row0 + r];
#pragma unroll
        for (int x = 0; x < 8; ++x) gwo[x] = fmaf(h[x], gt, gwo[x]);
      }
    }
    __syncthreads();
    // gW[a_, b] += sum_r Hprev[r, a_] * G_T[r, b]   (contracted over the 64 rows)
#pragma unroll
    for (int q = 0; q < M::NGW; ++q) {
      const int idx = wave + 4 * q;
      if (idx < M::NT * M::NT) {
        const int ta = idx / M::NT, tb = idx % M::NT;
        const bf16_t* ap = hpt + (ta * 32 + lane % 32) * M::PT + 8 * (lane / 32);
        const bf16_t* bp = gtt + (tb * 32 + lane % 32) * M::PT + 8 * (lane / 32);
#pragma unroll
        for (int ks = 0; ks < R / 16; ++ks) {
          const bf16x8 af = as_frag(*reinterpret_cast<const uint4*>(ap + ks * 16));
          const bf16x8 bf = as_frag(*reinterpret_cast<const uint4*>(bp + ks * 16));
          gw[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bf, gw[q], 0, 0, 0);
        }
      }
    }
    if (need_gh) {
      // G_Hprev[r, j] = sum_b G_T[r, b] * W[j, b]
      floatx16 acc[M::NTM];
      tile_product<D>(at, wfrag, tm0, acc);
      __syncthreads();  // all products done: at / gtt may be overwritten
      if (TO_EMBED) {
#pragma unroll
        for (int q = 0; q < M::NTM; ++q) {
          const int tm = tm0 + q * M::WPC;
          if (tm < M::MT) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int i = tm * 32 + (r / 4) * 8 + (lane / 32) * 4 + r % 4;
              stage[i * M::PO + tn * 32 + lane % 32] = acc[q][r];
            }
          }
        }
        __syncthreads();
        for (int idx = tid; idx < R * (D / 4); idx += kBlock) {
          const int r = idx / (D / 4), cc = (idx % (D / 4)) * 4;
          if (r >= nrows) continue;
          const float4 gq = *reinterpret_cast<const float4*>(stage + r * M::PO + cc);
          const size_t off = static_cast<size_t>(row0 + r) * D + cc;
          if (a.mode == EMBED_WRITE_GRAD) {
            *reinterpret_cast<float4*>(a.gE + off) = gq;
          } else {
            const float4 m0 = *reinterpret_cast<const float4*>(a.mE + off);
            const float4 v0 = *reinterpret_cast<const float4*>(a.vE + off);
            const float4 e0 = *reinterpret_cast<const float4*>(a.E + off);
            const float gv[4] = {gq.x, gq.y, gq.z, gq.w};
            const float mv[4] = {m0.x, m0.y, m0.z, m0.w};
            const float vv[4] = {v0.x, v0.y, v0.z, v0.w};
            const float ev[4] = {e0.x, e0.y, e0.z, e0.w};
            float mo[4], vo[4], eo[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
              mo[x] = a.adam.b1 * mv[x] + (1.f - a.adam.b1) * gv[x];
              vo[x] = a.adam.b2 * vv[x] + (1.f - a.adam.b2) * gv[x] * gv[x];
              const float upd = (mo[x] * a.adam.inv_bc1) / (sqrtf(vo[x]) * a.adam.inv_sqrt_bc2 + a.adam.eps);
              eo[x] = ev[x] - a.adam.lr * upd;
            }
            *reinterpret_cast<float4*>(a.mE + off) = make_float4(mo[0], mo[1], mo[2], mo[3]);
            *reinterpret_cast<float4*>(a.vE + off) = make_float4(vo[0], vo[1], vo[2], vo[3]);
            *reinterpret_cast<float4*>(a.E + off) = make_float4(eo[0], eo[1], eo[2], eo[3]);
            uint2 eb;
            eb.x = static_cast<uint32_t>(f32_to_bf16(eo[0])) | (static_cast<uint32_t>(f32_to_bf16(eo[1])) << 16);
            eb.y = static_cast<uint32_t>(f32_to_bf16(eo[2])) | (static_cast<uint32_t>(f32_to_bf16(eo[3])) << 16);
            *reinterpret_cast<uint2*>(static_cast<bf16_t*>(a.Eb) + off) = eb;
          }
        }
      } else {
        // GZ_out = G_Hprev * [Hprev > 0], staged in `at` as bf16 for 16-byte stores
#pragma unroll
        for (int q = 0; q < M::NTM; ++q) {
          const int tm = tm0 + q * M::WPC;
          if (tm < M::MT) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int i = tm * 32 + (r / 4) * 8 + (lane / 32) * 4 + r % 4;
              const int j = tn * 32 + lane % 32;
              const bf16_t h = hpt[j * M::PT + i];
              const bool pos = (h & 0x8000u) == 0 && (h & 0x7fffu) != 0;
              at[i * M::PA + j] = pos ? f32_to_bf16(acc[q][r]) : static_cast<bf16_t>(0);
            }
          }
        }
        __syncthreads();
        bf16_t* GZo = static_cast<bf16_t*>(a.GZ_out);
        for (int idx = tid; idx < R * M::LPR; idx += kBlock) {
          const int r = idx / M::LPR;
          if (r < nrows)
            *reinterpret_cast<uint4*>(GZo + static_cast<size_t>(row0 + r) * D + c0) =
                *reinterpret_cast<const uint4*>(at + r * M::PA + c0);
        }
      }
    }
    __syncthreads();
  }
  // weight-gradient partials of this workgroup
#pragma unroll
  for (int q = 0; q < M::NGW; ++q) {
    const int idx = wave + 4 * q;
    if (idx < M::NT * M::NT) {
      const int ta = idx / M::NT, tb = idx % M::NT;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int ai = ta * 32 + (r / 4) * 8 + (lane / 32) * 4 + r % 4;
        a.gW_partial[static_cast<size_t>(blockIdx.x) * D * D + ai * D + tb * 32 + lane % 32] = gw[q][r];
      }
    }
  }
  if (LAST) {
    constexpr int G = kBlock / M::LPR;
#pragma unroll
    for (int x = 0; x < 8; ++x) red[(tid / M::LPR) * D + c0 + x] = gwo[x];
    __syncthreads();
    if (tid < D) {
      float sacc = 0.f;
      for (int gq = 0; gq < G; ++gq) sacc += red[gq * D + tid];
      a.gwout_partial[static_cast<size_t>(blockIdx.x) * D + tid] = sacc;
    }
  }
}

template <typename K>
void allow_lds(K kernel, size_t bytes) {
  if (bytes > 48 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
}

template <int D>
void fwd_t(const Launch& ln, const GraphView& g, const void* X, const float* W, int w_stride, void* Y,
           const float* w_out, int wout_stride, float* t, float* heavy_partial) {
  if (g.num_chunks > 0) {
    ln.begin(KK_HEAVY);
    PlainSrc<bf16_t, D> src{static_cast<const bf16_t*>(X), g.sb};
    heavy_wide_kernel<bf16_t, D, PlainSrc<bf16_t, D>><<<g.num_chunks, kBlock, 0, ln.st>>>(g, src, heavy_partial);
    ln.end(KK_HEAVY);
  }
  allow_lds(fwd_hidden_bf16_kernel<D>, fwd_lds<D>());
  ln.begin(KK_FWD_HIDDEN);
  fwd_hidden_bf16_kernel<D><<<g.num_blocks, kBlock, fwd_lds<D>(), ln.st>>>(
      g, static_cast<const bf16_t*>(X), W, w_stride, static_cast<bf16_t*>(Y), w_out, wout_stride, t,
      heavy_partial);
  ln.end(KK_FWD_HIDDEN);
}

template <int D>
void bwd_t(const Launch& ln, bool last, bool to_embed, const GraphView& gt, const BwdArgs& a) {
  if (gt.num_chunks > 0) {
    ln.begin(KK_HEAVY);
    if (last) {
      LastSrc<bf16_t, D> src{static_cast<const bf16_t*>(a.Hcur), gt.sb, a.g_t, a.w_out, a.wout_stride, {}};
      heavy_wide_kernel<bf16_t, D, LastSrc<bf16_t, D>><<<gt.num_chunks, kBlock, 0, ln.st>>>(gt, src, a.heavy_partial);
    } else {
      PlainSrc<bf16_t, D> src{static_cast<const bf16_t*>(a.GZ_in), gt.sb};
      heavy_wide_kernel<bf16_t, D, PlainSrc<bf16_t, D>><<<gt.num_chunks, kBlock, 0, ln.st>>>(gt, src, a.heavy_partial);
    }
    ln.end(KK_HEAVY);
  }
  const int kind = to_embed ? KK_BWD_EMBED : KK_BWD_HIDDEN;
  ln.begin(kind);
#define GCO_BWD(L_, E_)                                                                         \
  {                                                                                             \
    allow_lds(bwd_hidden_bf16_kernel<D, L_, E_>, bwd_lds<D>());                                 \
    bwd_hidden_bf16_kernel<D, L_, E_><<<gt.num_blocks, kBlock, bwd_lds<D>(), ln.st>>>(gt, a);   \
  }
  if (last && to_embed) GCO_BWD(true, true)
  else if (last) GCO_BWD(true, false)
  else if (to_embed) GCO_BWD(false, true)
  else GCO_BWD(false, false)
#undef GCO_BWD
  ln.end(kind);
}

}  // namespace

void launch_fwd_hidden_bf16(const Launch& ln, int D, const GraphView& g, const void* X, const float* W,
                            int w_stride, void* Y, const float* w_out, int wout_stride, float* t,
                            float* heavy_partial) {
  switch (D) {
    case 32: fwd_t<32>(ln, g, X, W, w_stride, Y, w_out, wout_stride, t, heavy_partial); break;
    case 64: fwd_t<64>(ln, g, X, W, w_stride, Y, w_out, wout_stride, t, heavy_partial); break;
    case 128: fwd_t<128>(ln, g, X, W, w_stride, Y, w_out, wout_stride, t, heavy_partial); break;
    default: break;
  }
}

// `gt` is the view with the scale vectors exchanged (A_hat^T).
void launch_bwd_hidden_bf16(const Launch& ln, int D, bool last, bool to_embed, const GraphView& gt,
                            const BwdArgs& a) {
  switch (D) {
    case 32: bwd_t<32>(ln, last, to_embed, gt, a); break;
    case 64: bwd_t<64>(ln, last, to_embed, gt, a); break;
    case 128: bwd_t<128>(ln, last, to_embed, gt, a); break;
    default: break;
  }
}

}  // namespace gco
