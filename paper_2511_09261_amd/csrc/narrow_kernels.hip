// Width-1 kernels: the scalar layer's aggregation z = A_hat t with the sigmoid (Eq. 4),
// the loss with its derivative (Eq. 5) and the first backward aggregation g_t = A_hat^T g_z.
//
// All three are sums over the entries of each row of one gathered scalar.  They run on
// the light stream (per row its diagonal entry, then its neighbours; rows with very many
// neighbours hold only the diagonal entry): a wavefront owns a contiguous run of rows of
// one subgraph, cut on the host so that all wavefronts carry about the same number of
// entries, and consumes the stream 64 entries at a time, one entry per lane, whatever
// the row lengths:
//   * the entries of the next step and the gathered values of this step are requested
//     before the current step is reduced;
//   * the rows that begin in the step mark their first entry (an LDS scatter of the row
//     number), an inclusive max-scan over the lanes gives every entry its row, a segmented
//     inclusive sum gives the last lane of every row the row's share of the step, which
//     it adds to the row's accumulator in LDS -- one lane per row and step, steps in
//     order: a fixed order;
//   * at the end the lanes turn into rows and apply the row-wise epilogue.
// Rows with very many neighbours are summed by one workgroup each (the first workgroups
// of the grid), which also applies their epilogue; the stream part skips those rows.
#include "device_utils.h"
#include "gco_internal.h"

namespace gco {
namespace {

constexpr int kWaves = kBlock / 64;
constexpr int kBatchRows = 512;  // rows whose offsets and sums a wavefront keeps in LDS at a time

// Sum of v over the workgroup in a fixed order; every thread gets the total.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  if (threadIdx.x % 64 == 0) red[threadIdx.x / 64] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) s += red[w];
  __syncthreads();
  return s;
}

// Cross-lane moves on the data-parallel-primitive path (no LDS): lane l receives the value
// of lane l - N of its 16-lane row (row_shr:N), or rows 1 and 3 receive lane 15 of the row
// before them (row_bcast:15), or rows 2 and 3 receive lane 31 (row_bcast:31); every lane
// without a source keeps `fill`.  The six moves N = 1, 2, 4, 8, bcast 15, bcast 31 make an
// inclusive scan over the 64 lanes.
template <int kCtrl, int kRowMask>
__device__ __forceinline__ int dpp_move(int fill, int v) {
  return __builtin_amdgcn_update_dpp(fill, v, kCtrl, kRowMask, 0xf, false);
}
template <int kCtrl, int kRowMask>
__device__ __forceinline__ float dpp_move(float fill, float v) {
  return __int_as_float(
      __builtin_amdgcn_update_dpp(__float_as_int(fill), __float_as_int(v), kCtrl, kRowMask, 0xf, false));
}
#define GCO_SCAN_STEPS(STEP) \
  STEP(0x111, 0xf) STEP(0x112, 0xf) STEP(0x114, 0xf) STEP(0x118, 0xf) STEP(0x142, 0xa) STEP(0x143, 0xc)

// Inclusive running maximum over the lanes (values >= -1).
__device__ __forceinline__ int scan_max(int v) {
#define GCO_STEP(C, M) v = max(v, dpp_move<C, M>(-1, v));
  GCO_SCAN_STEPS(GCO_STEP)
#undef GCO_STEP
  return v;
}

// Inclusive sum over the lanes, restarted wherever key changes (equal keys are contiguous).
__device__ __forceinline__ float scan_sum_by_key(float v, int key) {
#define GCO_STEP(C, M)                            \
  {                                               \
    const float ov = dpp_move<C, M>(0.f, v);      \
    const int ok = dpp_move<C, M>(-2, key);       \
    if (ok == key) v += ov;                       \
  }
  GCO_SCAN_STEPS(GCO_STEP)
#undef GCO_STEP
  return v;
}

// What differs between the three kernels.
//   gather(j)        the scalar of column j
//   kWeighted        entries count with their A_hat value and the diagonal entry takes
//                    part; otherwise every neighbour counts 1 and the diagonal entry 0
//   finish(i, s, ls) row i has the sum s; ls accumulates the lane's loss terms
struct ReadoutOp {  // z = A_hat t, p = sigmoid(z)
  static constexpr bool kWeighted = true;
  const float* __restrict__ t;
  float* __restrict__ z;
  float* __restrict__ p;
  __device__ __forceinline__ float gather(int j) const { return t[j]; }
  __device__ __forceinline__ void finish(int i, float s, double&) const {
    z[i] = s;
    p[i] = 1.f / (1.f + expf(-s));
  }
};
struct BackOp {  // g_t = A_hat^T g_z (the view passed in holds the transposed stream)
  static constexpr bool kWeighted = true;
  const float* __restrict__ g_z;
  float* __restrict__ g_t;
  __device__ __forceinline__ float gather(int j) const { return g_z[j]; }
  __device__ __forceinline__ void finish(int i, float s, double&) const { g_t[i] = s; }
};
struct LossOp {  // s = A_loc p; g_z = (c + q s) p (1 - p); loss term p (c + q/2 s)
  static constexpr bool kWeighted = false;
  const float* __restrict__ p;
  const float* __restrict__ cl;
  float q;
  float* __restrict__ g_z;
  __device__ __forceinline__ float gather(int j) const { return p[j]; }
  __device__ __forceinline__ void finish(int i, float s, double& ls) const {
    const float pi = p[i], ci = cl[i];
    g_z[i] = (ci + q * s) * pi * (1.f - pi);
    ls += static_cast<double>(pi) *
          (static_cast<double>(ci) + 0.5 * static_cast<double>(q) * static_cast<double>(s));
  }
};

// Grid: g.num_heavy workgroups for the rows with very many neighbours, then the stream
// workgroups of decomposition WM_NARROW.  loss_partial (LossOp only) gets one value per
// workgroup of the grid.
template <class Op>
__global__ __launch_bounds__(kBlock) void narrow_stream_kernel(GraphView g, Op op,
                                                               double* __restrict__ loss_partial) {
  __shared__ float red[kWaves];
  __shared__ double dred[kWaves];
  __shared__ int mark_s[kWaves][64];
  __shared__ int rp_s[kWaves][kBatchRows + 1];
  __shared__ float rowacc_s[kWaves][kBatchRows];
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  double lsum = 0.0;

  if (static_cast<int>(blockIdx.x) < g.num_heavy) {
    // one row with very many neighbours: CSR entries {column, A_hat value};
    // 32 entries per thread and pass: first all entries, then all gathered values
    const int i = g.heavy_rows[blockIdx.x];
    if (i < 0) return;  // the row's subgraph sits out
    const int e0 = g.rowptr[i], e1 = g.rowptr[i + 1];
    constexpr int kU = 32;
    float acc = 0.f;
    for (int e = e0 + tid; e < e1; e += kU * kBlock) {
      int2 en[kU];
      float v[kU];
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        const int ee = e + u * kBlock;
        en[u] = ee < e1 ? g.ent[ee] : make_int2(i, 0);
      }
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        const float x = op.gather(en[u].x);
        v[u] = e + u * kBlock < e1 ? (Op::kWeighted ? __int_as_float(en[u].y) * x : x) : 0.f;
      }
#pragma unroll
      for (int w = 1; w < kU; w *= 2)
#pragma unroll
        for (int u = 0; u < kU; u += 2 * w) v[u] += v[u + w];
      acc += v[0];
    }
    float total = block_sum(acc, red);
    if (tid == 0) {
      if (Op::kWeighted) total += g.diag[i] * op.gather(i);
      op.finish(i, total, lsum);
      if (loss_partial != nullptr) loss_partial[blockIdx.x] = lsum;
    }
    return;
  }

  const int b = blockIdx.x - g.num_heavy;
  const int k = g.wblk_k[WM_NARROW][b];
  if (k < 0) return;
  const WaveRun run = g.wave_runs[WM_NARROW][b * kWaves + wave];
  const int r0 = run.rbeg + run.tile0 * kWaveRows, r1 = min(run.rend, run.rbeg + run.tile1 * kWaveRows);
  int* mark = mark_s[wave];
  int* rp = rp_s[wave];
  float* rowacc = rowacc_s[wave];

  for (int rb = r0; rb < r1; rb += kBatchRows) {
    // a batch of rows: their stream offsets and accumulators live in LDS
    const int nr = min(kBatchRows, r1 - rb);
    for (int q = lane; q <= nr; q += 64) rp[q] = g.wrowptr[rb + q];
    for (int q = lane; q < nr; q += 64) rowacc[q] = 0.f;
    const int eb = g.wrowptr[rb], ee = g.wrowptr[rb + nr];
    wave_lds_handoff();
    int first = 0;   // first row of the batch whose entries have not begun yet
    int carry = -1;  // the row that runs on from the previous step
    // software pipeline: entries two steps ahead, gathered values one step ahead
    int col_cur = 0, col_nxt = 0;
    float w_cur = 0.f, w_nxt = 0.f, x_cur = 0.f;
    if (eb + lane < ee) {
      col_cur = g.went[eb + lane].x;
      if (Op::kWeighted) w_cur = g.wval[eb + lane];
      x_cur = op.gather(col_cur);
    }
    if (eb + 64 + lane < ee) {
      col_nxt = g.went[eb + 64 + lane].x;
      if (Op::kWeighted) w_nxt = g.wval[eb + 64 + lane];
    }
    for (int e0 = eb; e0 < ee; e0 += 64) {
      int col_nn = 0;
      float w_nn = 0.f, x_nxt = 0.f;
      if (e0 + 128 + lane < ee) {
        col_nn = g.went[e0 + 128 + lane].x;
        if (Op::kWeighted) w_nn = g.wval[e0 + 128 + lane];
      }
      if (e0 + 64 + lane < ee) x_nxt = op.gather(col_nxt);
      // Which row every entry of the step belongs to.  Every row has at least one entry,
      // so at most 64 rows begin in the step: rows first, first + 1, ...
      mark[lane] = -1;
      const int myrow = first + lane;
      const int myrp = myrow < nr ? rp[myrow] : ee;
      const bool begins = myrow < nr && myrp < e0 + 64;
      wave_lds_handoff();
      if (begins) mark[myrp - e0] = myrow;
      first += __builtin_popcountll(__ballot(begins));
      wave_lds_handoff();
      int row = mark[lane];
      const bool is_start = row >= 0;
      row = scan_max(row);
      if (row < 0) row = carry;
      // the row's share of the step, at the row's last lane
      float v = 0.f;
      if (e0 + lane < ee) v = Op::kWeighted ? w_cur * x_cur : (is_start ? 0.f : x_cur);
      v = scan_sum_by_key(v, row);
      const int next_row = __shfl_down(row, 1, 64);
      if ((lane == 63 || next_row != row) && row >= 0) rowacc[row] += v;
      wave_lds_handoff();
      carry = __builtin_amdgcn_readlane(row, 63);
      col_cur = col_nxt; w_cur = w_nxt; x_cur = x_nxt;
      col_nxt = col_nn; w_nxt = w_nn;
    }
    for (int q = lane; q < nr; q += 64) {
      const int i = rb + q;
      const bool heavy = g.num_heavy > 0 && g.heavy_of_row[i] >= 0;
      if (!heavy) op.finish(i, rowacc[q], lsum);
    }
    wave_lds_handoff();
  }
  if (loss_partial != nullptr) {
    lsum = wave_sum(lsum);
    if (lane == 0) dred[wave] = lsum;
    __syncthreads();
    if (tid == 0) loss_partial[g.num_heavy + b] = ((dred[0] + dred[1]) + dred[2]) + dred[3];
  }
}

template <class Op>
void launch_narrow(const Launch& ln, int kind, const GraphView& g, const Op& op, double* loss_partial) {
  ln.begin(kind);
  narrow_stream_kernel<Op><<<g.num_heavy + g.num_wblocks[WM_NARROW], kBlock, 0, ln.st>>>(g, op, loss_partial);
  ln.end(kind);
}

}  // namespace

void launch_fwd_readout(const Launch& ln, const GraphView& g, const float* t, float* z, float* p) {
  launch_narrow(ln, KK_FWD_READOUT, g, ReadoutOp{t, z, p}, nullptr);
}

void launch_loss(const Launch& ln, const GraphView& g, const float* p, const float* c, float q, float* g_z,
                 double* loss_partial) {
  launch_narrow(ln, KK_LOSS, g, LossOp{p, c, q, g_z}, loss_partial);
}

void launch_bwd_readout(const Launch& ln, const GraphView& g, const float* g_z, float* g_t) {
  launch_narrow(ln, KK_BWD_READOUT, transposed(g), BackOp{g_z, g_t}, nullptr);
}

}  // namespace gco
