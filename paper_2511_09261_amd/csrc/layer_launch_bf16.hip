// bf16-storage hidden layers (widths 64 and 128): the order of launches around the
// wave-per-tile kernels of wave_kernels_bf16.hip, and the chunked pre-reduction of rows
// with very many neighbours that precedes each aggregation.
#include "bf16_common.h"
#include "device_utils.h"
#include "gco_internal.h"

namespace gco {
namespace {

// Chunked pre-reduction of very long rows: partial[c, :] = sum over the entries e of chunk c
// of A_hat value(e) * X[column(e), :], fp32.  A workgroup per chunk: lane group grp (the
// lanes that share one 16-byte slice per lane of a feature row) takes entries grp, grp + G,
// ..., four loads in flight; the G group sums are added in order.
template <int D>
__global__ __launch_bounds__(kBlock) void heavy_wide_b_kernel(GraphView g, const bf16_t* __restrict__ X,
                                                              float* __restrict__ partial) {
  constexpr int LPR = D / 8;       // lanes per feature row (16 bytes each)
  constexpr int G = kBlock / LPR;  // lane groups per workgroup
  __shared__ float red[kBlock * 8];
  const int ch = blockIdx.x;
  const int tid = threadIdx.x;
  const int grp = tid / LPR, c0 = (tid % LPR) * 8;
  if (g.chunk_part[ch] < 0) return;  // the row's subgraph sits out
  float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const int eb = g.chunk_end[ch];
  for (int e = g.chunk_begin[ch] + grp; e < eb; e += 4 * G) {
    uint4 rw[4];
    float s4[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int ee = e + x * G;
      rw[x] = make_uint4(0u, 0u, 0u, 0u);
      s4[x] = 0.f;
      if (ee < eb) {
        const int2 en = g.ent[ee];
        rw[x] = *reinterpret_cast<const uint4*>(X + static_cast<size_t>(en.x) * D + c0);
        s4[x] = __int_as_float(en.y);
      }
    }
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      float v[8];
      unpack8(rw[x], v);
#pragma unroll
      for (int y = 0; y < 8; ++y) a8[y] = fmaf(s4[x], v[y], a8[y]);
    }
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

template <int D>
void pre_reduce(const Launch& ln, const GraphView& g, const void* X, float* heavy_partial) {
  if (g.num_chunks == 0) return;
  ln.begin(KK_HEAVY);
  heavy_wide_b_kernel<D><<<g.num_chunks, kBlock, 0, ln.st>>>(g, static_cast<const bf16_t*>(X), heavy_partial);
  ln.end(KK_HEAVY);
}

template <int D>
void fwd_t(const Launch& ln, const GraphView& g, const void* X, const float* W, int w_stride, void* Y,
           const float* w_out, int wout_stride, float* t, float* heavy_partial) {
  pre_reduce<D>(ln, g, X, heavy_partial);
  launch_fwd_hidden_wave(ln, D, g, X, W, w_stride, Y, w_out, wout_stride, t, heavy_partial);
}

template <int D>
void bwd_t(const Launch& ln, bool last, bool to_embed, const GraphView& gt, const BwdArgs& a) {
  BwdArgs b = a;
  if (last) {  // G_Z of the last hidden layer is formed first
    launch_form_gz_last(ln, D, gt, a);
    b.GZ_in = a.GZ_last;
  }
  pre_reduce<D>(ln, gt, b.GZ_in, a.heavy_partial);
  launch_bwd_hidden_wave(ln, D, to_embed, gt, b);
}

}  // namespace

void launch_fwd_hidden_bf16(const Launch& ln, int D, const GraphView& g, const void* X, const float* W,
                            int w_stride, void* Y, const float* w_out, int wout_stride, float* t,
                            float* heavy_partial) {
  switch (D) {
    case 64: fwd_t<64>(ln, g, X, W, w_stride, Y, w_out, wout_stride, t, heavy_partial); break;
    case 128: fwd_t<128>(ln, g, X, W, w_stride, Y, w_out, wout_stride, t, heavy_partial); break;
    default: break;
  }
}

// `gt` is the view with the scale vectors exchanged (A_hat^T).
void launch_bwd_hidden_bf16(const Launch& ln, int D, bool last, bool to_embed, const GraphView& gt,
                            const BwdArgs& a) {
  switch (D) {
    case 64: bwd_t<64>(ln, last, to_embed, gt, a); break;
    case 128: bwd_t<128>(ln, last, to_embed, gt, a); break;
    default: break;
  }
}

}  // namespace gco
