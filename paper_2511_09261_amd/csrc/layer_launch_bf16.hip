// bf16-storage hidden layers (widths 64 and 128): the order of launches around the
// wave-per-tile kernels of wave_kernels_bf16.hip, and the chunked pre-reduction of rows
// with very many neighbours that precedes each aggregation.
#include "bf16_common.h"
#include "device_utils.h"
#include "gco_internal.h"
#include "heavy_chunk.h"

namespace gco {
namespace {

// Chunked pre-reduction of very long rows as a launch of its own: a workgroup per chunk.
template <int D>
__global__ __launch_bounds__(kBlock) void heavy_wide_b_kernel(GraphView g, const bf16_t* __restrict__ X,
                                                              float* __restrict__ partial) {
  __shared__ float red[kBlock * 8];
  const int ch = blockIdx.x;
  if (g.chunk_part[ch] < 0) return;  // the row's subgraph sits out
  reduce_chunk<D>(g, ChunkPlainRows<D>{X}, partial, ch, red);
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
           const float* w_out, int wout_stride, float* t, float* heavy_partial, bool partial_ready) {
  if (!partial_ready) pre_reduce<D>(ln, g, X, heavy_partial);
  launch_fwd_hidden_wave(ln, D, g, X, W, w_stride, Y, w_out, wout_stride, t, heavy_partial);
}

template <int D>
void bwd_t(const Launch& ln, bool last, bool to_embed, const GraphView& gt, const BwdArgs& a) {
  BwdArgs b = a;
  if (last) {
    // G_Z of the last hidden layer is formed first; the same launch carries the chunks of the
    // pre-reduction as extra workgroups (they form the rows they need on the fly)
    launch_form_gz_last(ln, D, gt, a);
    b.GZ_in = a.GZ_last;
  } else {
    pre_reduce<D>(ln, gt, b.GZ_in, a.heavy_partial);
  }
  launch_bwd_hidden_wave(ln, D, to_embed, gt, b);
}

}  // namespace

void launch_fwd_hidden_bf16(const Launch& ln, int D, const GraphView& g, const void* X, const float* W,
                            int w_stride, void* Y, const float* w_out, int wout_stride, float* t,
                            float* heavy_partial, bool partial_ready) {
  switch (D) {
    case 64: fwd_t<64>(ln, g, X, W, w_stride, Y, w_out, wout_stride, t, heavy_partial, partial_ready); break;
    case 128: fwd_t<128>(ln, g, X, W, w_stride, Y, w_out, wout_stride, t, heavy_partial, partial_ready); break;
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
