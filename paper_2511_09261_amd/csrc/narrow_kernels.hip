// Width-1 kernels: the scalar layer's aggregation z = A_hat t with the sigmoid (Eq. 4),
// the loss with its derivative (Eq. 5) and the first backward aggregation g_t = A_hat^T g_z.
//
// All three are sums over the entries of each row of one gathered scalar.  They run on
// the light stream (per row its diagonal entry, then its neighbours; rows with very many
// neighbours hold only the diagonal entry), which also names the row of every entry: a
// wavefront owns a contiguous run of rows of one subgraph, cut on the host so that all
// wavefronts carry about the same number of entries, and consumes its range of the stream
// 64 entries at a time, one entry per lane, whatever the row lengths:
//   * three groups of K steps are under way at any time: one is reduced, the scalars of
//     the next are being gathered, the entries of the one after are being read;
//   * a segmented inclusive sum keyed by the row number (data-parallel-primitive moves,
//     no LDS) gives the last lane of every row the row's share of the step; a row that runs
//     on into the next step hands its partial sum over in a scalar register; the last lane
//     of a row applies the row-wise epilogue.  One fixed order of additions.
// Rows with very many neighbours are summed by a whole workgroup each, which also applies
// their epilogue; the stream skips them (their row number reads -2).
//
// Two launch forms: three separate kernels over a common decomposition (any graph), or
// ONE launch with a workgroup per subgraph that keeps the subgraph's vectors in LDS (when
// they fit).
#include "device_utils.h"
#include "gco_internal.h"

namespace gco {
namespace {

constexpr int kWaves = kBlock / 64;

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
//   finish(i, s, ls, y) row i has the sum s; ls accumulates the lane's loss terms; y is what
//                   row_inputs(i) returned earlier
//   row_inputs(i)   values of row i that the epilogue needs, requested together with the
//                   gathered scalars, so that the epilogue itself loads nothing (a load there
//                   would have to wait behind the entries requested ahead: vector memory
//                   operations complete in order); kRowInputs says whether there are any
struct ReadoutOp {  // z = A_hat t, p = sigmoid(z)
  static constexpr bool kWeighted = true;
  const float* __restrict__ t;
  float* __restrict__ z;
  float* __restrict__ p;
  __device__ __forceinline__ const float* source() const { return t; }
  __device__ __forceinline__ float gather(int j) const { return t[j]; }
  static constexpr bool kRowInputs = false;
  __device__ __forceinline__ float2 row_inputs(int) const { return make_float2(0.f, 0.f); }
  __device__ __forceinline__ void finish(int i, float s, double&, float2) const {
    z[i] = s;
    p[i] = 1.f / (1.f + expf(-s));
  }
};
struct BackOp {  // g_t = A_hat^T g_z (the view passed in holds the transposed stream)
  static constexpr bool kWeighted = true;
  const float* __restrict__ g_z;
  float* __restrict__ g_t;
  __device__ __forceinline__ const float* source() const { return g_z; }
  __device__ __forceinline__ float gather(int j) const { return g_z[j]; }
  static constexpr bool kRowInputs = false;
  __device__ __forceinline__ float2 row_inputs(int) const { return make_float2(0.f, 0.f); }
  __device__ __forceinline__ void finish(int i, float s, double&, float2) const { g_t[i] = s; }
};
struct LossOp {  // s = A_loc p; g_z = (c + q s) p (1 - p); loss term p (c + q/2 s)
  static constexpr bool kWeighted = false;
  const float* __restrict__ p;
  const float* __restrict__ cl;
  float q;
  float* __restrict__ g_z;
  __device__ __forceinline__ const float* source() const { return p; }
  __device__ __forceinline__ float gather(int j) const { return p[j]; }
  static constexpr bool kRowInputs = true;
  __device__ __forceinline__ float2 row_inputs(int i) const { return make_float2(p[i], cl[i]); }
  __device__ __forceinline__ void finish(int i, float s, double& ls, float2 y) const {
    const float pi = y.x, ci = y.y;
    g_z[i] = (ci + q * s) * pi * (1.f - pi);
    ls += static_cast<double>(pi) *
          (static_cast<double>(ci) + 0.5 * static_cast<double>(q) * static_cast<double>(s));
  }
};

// One wavefront sums the rows whose entries fill [E0, E1) of the light stream (went, wval,
// wrowid): whole rows, in order.  K = steps of 64 entries requested at a time.  `between`
// runs once, after the first entries have been requested and before anything is gathered.
struct NothingBetween {
  __device__ __forceinline__ void operator()() const {}
};
template <class Op, int K, class Between = NothingBetween>
__device__ __forceinline__ void stream_rows(const int2* __restrict__ went, const float* __restrict__ wval,
                                            const int* __restrict__ wrowid, const Op& op, int E0, int E1,
                                            double& lsum, Between&& between = NothingBetween{}) {
  const int lane = threadIdx.x % 64;
  // K steps of the stream: column, row and value of this lane's entry, and the gathered scalar
  struct Group {
    int col[K], row[K];
    float w[K], x[K];
    float2 y[K];  // row_inputs of the entry's row (unused and removed where the operation has none)
  };
  auto request = [&](int base, Group& s) {
#pragma unroll
    for (int u = 0; u < K; ++u) {
      const int idx = base + 64 * u + lane;
      const bool ok = idx < E1;
      s.col[u] = ok ? went[idx].x : 0;
      s.row[u] = ok ? wrowid[idx] : -1;
      s.w[u] = (ok && Op::kWeighted) ? wval[idx] : 0.f;
    }
  };
  // lanes past the range (row number -1) gather nothing
  auto gather = [&](Group& s) {
#pragma unroll
    for (int u = 0; u < K; ++u) {
      s.x[u] = 0.f;
      if (s.row[u] != -1) s.x[u] = op.gather(s.col[u]);
      if (Op::kRowInputs) {
        s.y[u] = make_float2(0.f, 0.f);
        if (s.row[u] >= 0) s.y[u] = op.row_inputs(s.row[u]);
      }
    }
  };
  int carry_row = -1;     // the row that runs on from the previous step, and its sum so far
  float carry_sum = 0.f;
  // the K steps of one group; nrow0 = this lane's row in the first step of the group after it
  auto reduce_group = [&](int g0, const Group& s, int nrow0) {
#pragma unroll
    for (int u = 0; u < K; ++u) {
      const int e0 = g0 + 64 * u;
      if (e0 < E1) {
        const int nrow = u + 1 < K ? s.row[(u + 1) % K] : nrow0;
        const int next_first = __builtin_amdgcn_readfirstlane(nrow);  // -1 past the range
        const int row = s.row[u];
        const bool valid = row >= 0;  // inside the range and not the entry of a pre-reduced row
        float v = 0.f;
        // the diagonal entry is the one whose column is the row itself (no self loops)
        if (valid) v = Op::kWeighted ? s.w[u] * s.x[u] : (s.col[u] == row ? 0.f : s.x[u]);
        v = scan_sum_by_key(v, row);
        int next_row = __shfl_down(row, 1, 64);
        if (lane == 63) next_row = next_first;
        const float total = v + (row == carry_row ? carry_sum : 0.f);
        if (valid && next_row != row) op.finish(row, total, lsum, s.y[u]);
        const int row63 = __builtin_amdgcn_readlane(row, 63);
        const float tot63 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(total), 63));
        const bool runs_on = row63 >= 0 && next_first == row63;
        carry_row = runs_on ? row63 : -1;
        carry_sum = runs_on ? tot63 : 0.f;
      }
    }
  };
  // Three groups of registers take turns: while one is reduced, the scalars of the next are
  // being gathered (its entries arrived a group ago) and the entries of the one after are
  // being read.  Every load of a group is issued a whole group of steps before it is used.
  Group a, b, c;
  request(E0, a);
  request(E0 + 64 * K, b);
  between();  // what has to happen before the first gather, while the first entries travel
  gather(a);
  for (int g0 = E0; g0 < E1; g0 += 192 * K) {
    request(g0 + 128 * K, c);
    gather(b);
    reduce_group(g0, a, b.row[0]);
    if (g0 + 64 * K >= E1) break;
    request(g0 + 192 * K, a);
    gather(c);
    reduce_group(g0 + 64 * K, b, c.row[0]);
    if (g0 + 128 * K >= E1) break;
    request(g0 + 256 * K, b);
    gather(a);
    reduce_group(g0 + 128 * K, c, a.row[0]);
  }
}

// CSR entries e0 .. e1 of one row with very many neighbours, summed by the whole workgroup
// (NT threads): entries {column, A_hat value} of `ent`; kU entries per thread and pass: first
// all entries, then all gathered values.  Every thread returns the sum; red holds NT / 64
// floats.  Contains workgroup barriers.
template <class Op, int NT>
__device__ __forceinline__ float heavy_range_sum(const int2* __restrict__ ent, const Op& op, int i, int e0, int e1,
                                                 float* red) {
  const int tid = threadIdx.x;
  constexpr int kU = NT >= 1024 ? 8 : 32;
  float acc = 0.f;
  for (int e = e0 + tid; e < e1; e += kU * NT) {
    int2 en[kU];
    float v[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const int ee = e + u * NT;
      en[u] = ee < e1 ? ent[ee] : make_int2(i, 0);
    }
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const float x = op.gather(en[u].x);
      v[u] = e + u * NT < e1 ? (Op::kWeighted ? __int_as_float(en[u].y) * x : x) : 0.f;
    }
#pragma unroll
    for (int w = 1; w < kU; w *= 2)
#pragma unroll
      for (int u = 0; u < kU; u += 2 * w) v[u] += v[u + w];
    acc += v[0];
  }
  acc = wave_sum(acc);
  if (tid % 64 == 0) red[tid / 64] = acc;
  __syncthreads();
  float total = 0.f;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) total += red[w];
  __syncthreads();
  return total;
}

// The whole row i (diagonal included for the weighted operations).
template <class Op, int NT>
__device__ __forceinline__ float heavy_row_sum(const GraphView& g, const int2* __restrict__ ent, const Op& op,
                                               int i, float* red) {
  float total = heavy_range_sum<Op, NT>(ent, op, i, g.rowptr[i], g.rowptr[i + 1], red);
  if (Op::kWeighted) total += g.diag[i] * op.gather(i);
  return total;
}

// Grid: g.num_hparts workgroups for the rows with very many neighbours, then the stream
// workgroups of decomposition WM_NARROW.  A row with very many neighbours is summed in
// parts of kNarrowPartChunks chunks, a workgroup each, so that the longest row does not
// outlast the rest of the launch on a single compute unit; the workgroup that completes
// the row's count adds the parts in order and applies the row's epilogue (no workgroup
// waits for another).  loss_partial (LossOp only) gets one value per such row and one per
// stream workgroup.
template <class Op>
__global__ __launch_bounds__(kBlock) void narrow_stream_kernel(GraphView g, Op op,
                                                               double* __restrict__ loss_partial) {
  __shared__ float red[kWaves];
  __shared__ double dred[kWaves];
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  double lsum = 0.0;

  if (static_cast<int>(blockIdx.x) < g.num_hparts) {
    const int2 pt = g.hpart[blockIdx.x];
    const int h = pt.x, j = pt.y;
    const int i = g.heavy_rows[h];
    if (i < 0) return;  // the row's subgraph sits out
    const int c0 = g.heavy_chunk_ptr[h] + j * kNarrowPartChunks;
    const int c1 = min(c0 + kNarrowPartChunks, g.heavy_chunk_ptr[h + 1]);
    float total = heavy_range_sum<Op, kBlock>(g.ent, op, i, g.chunk_begin[c0], g.chunk_end[c1 - 1], red);
    if (tid == 0) {
      const int p0 = g.hpart_ptr[h], parts = g.hpart_ptr[h + 1] - p0;
      bool last = true;
      if (parts > 1) {
        g.hpart_partial[p0 + j] = total;
        __threadfence();  // the part is visible before the count says so
        last = atomicAdd(&g.hpart_count[h], 1) == parts - 1;
        if (last) {
          __threadfence();
          total = 0.f;
          for (int q = 0; q < parts; ++q)
            total += __hip_atomic_load(&g.hpart_partial[p0 + q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          g.hpart_count[h] = 0;  // ready for the next launch on this stream
        }
      }
      if (last) {
        if (Op::kWeighted) total += g.diag[i] * op.gather(i);
        op.finish(i, total, lsum, op.row_inputs(i));
        if (loss_partial != nullptr) loss_partial[h] = lsum;
      }
    }
    return;
  }

  const int b = blockIdx.x - g.num_hparts;
  const int k = g.wblk_k[WM_NARROW][b];
  if (k < 0) return;
  const WaveRun run = g.wave_runs[WM_NARROW][b * kWaves + wave];
  stream_rows<Op, 4>(g.went, g.wval, g.wrowid, op, run.e0, run.e1, lsum);
  if (loss_partial != nullptr) {
    lsum = wave_sum(lsum);
    if (lane == 0) dred[wave] = lsum;
    __syncthreads();
    if (tid == 0) loss_partial[g.num_heavy + b] = ((dred[0] + dred[1]) + dred[2]) + dred[3];
  }
}

// ---------------------------------------------------------------------------
// The three width-1 passes of a subgraph in ONE launch: read-out (Eq. 4), loss with its
// derivative (Eq. 5) and the backward aggregation of the scalar layer.  Subgraphs are
// independent (Sec. 3.3), so the only dependencies are inside a subgraph: one workgroup
// of NW wavefronts per subgraph keeps the subgraph's vectors in LDS (bufA: t, then dL/dz;
// bufB: p) and separates the passes by workgroup barriers.  Each wavefront sums a
// contiguous range of the subgraph's rows (cut on the host into equal shares of entries)
// with the stream routine above (cuts[k * NW + w] = its range of the light stream); rows
// with very many neighbours are summed by the whole workgroup after each pass.  `passes` = 1 stops after the probabilities, 2 after the loss.
// ---------------------------------------------------------------------------
struct FusedReadoutOp {
  static constexpr bool kWeighted = true;
  const float* bufA;   // t of the subgraph's rows
  float* bufB;         // p
  float* __restrict__ p;
  int rbeg;
  __device__ __forceinline__ float gather(int j) const { return bufA[j - rbeg]; }
  static constexpr bool kRowInputs = false;
  __device__ __forceinline__ float2 row_inputs(int) const { return make_float2(0.f, 0.f); }
  __device__ __forceinline__ void finish(int i, float s, double&, float2) const {
    const float pi = 1.f / (1.f + expf(-s));
    bufB[i - rbeg] = pi;
    p[i] = pi;
  }
};
struct FusedLossOp {
  static constexpr bool kWeighted = false;
  const float* bufB;   // p
  float* bufA;         // in: the linear coefficient c of the row; out: dL/dz
  float q;
  int rbeg;
  __device__ __forceinline__ float gather(int j) const { return bufB[j - rbeg]; }
  static constexpr bool kRowInputs = false;  // the epilogue reads LDS only
  __device__ __forceinline__ float2 row_inputs(int) const { return make_float2(0.f, 0.f); }
  __device__ __forceinline__ void finish(int i, float s, double& ls, float2) const {
    const float pi = bufB[i - rbeg], ci = bufA[i - rbeg];
    bufA[i - rbeg] = (ci + q * s) * pi * (1.f - pi);
    ls += static_cast<double>(pi) *
          (static_cast<double>(ci) + 0.5 * static_cast<double>(q) * static_cast<double>(s));
  }
};
struct FusedBackOp {
  static constexpr bool kWeighted = true;
  const float* bufA;   // dL/dz
  float* __restrict__ g_t;
  int rbeg;
  __device__ __forceinline__ float gather(int j) const { return bufA[j - rbeg]; }
  static constexpr bool kRowInputs = false;
  __device__ __forceinline__ float2 row_inputs(int) const { return make_float2(0.f, 0.f); }
  __device__ __forceinline__ void finish(int i, float s, double&, float2) const { g_t[i] = s; }
};

template <int NW>
__global__ __launch_bounds__(64 * NW) void scalar_layer_fused_kernel(
    GraphView g, const int2* __restrict__ cuts, const int* __restrict__ heavy_ptr, int cap,
    const float* __restrict__ t, float* __restrict__ p, const float* __restrict__ cl, float q,
    float* __restrict__ g_t, double* __restrict__ loss_partial, int passes) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* bufA = reinterpret_cast<float*>(smem);
  float* bufB = bufA + cap;
  float* red = bufB + cap;
  double* dred = reinterpret_cast<double*>(red + NW + (NW % 2));
  const int k = blockIdx.x;
  if (g.loss_ptr[k + 1] == g.loss_ptr[k]) return;  // the subgraph sits out
  const int tid = threadIdx.x, lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int rbeg = g.part_rows[k], rend = g.part_rows[k + 1];
  const int2 mine = cuts[k * NW + wave];  // this wavefront's range of the light stream
  const int h0 = heavy_ptr[k], h1 = heavy_ptr[k + 1];
  double lsum = 0.0;

  for (int r = rbeg + tid; r < rend; r += 64 * NW) bufA[r - rbeg] = t[r];
  __syncthreads();
  {
    const FusedReadoutOp op{bufA, bufB, p, rbeg};
    stream_rows<FusedReadoutOp, 8>(g.went, g.wval, g.wrowid, op, mine.x, mine.y, lsum);
    for (int hh = h0; hh < h1; ++hh) {
      const int i = g.heavy_rows[hh];
      const float total = heavy_row_sum<FusedReadoutOp, 64 * NW>(g, g.ent, op, i, red);
      if (tid == 0) op.finish(i, total, lsum, op.row_inputs(i));
    }
  }
  if (passes < 2) return;
  __syncthreads();
  // t has served; its place takes the linear coefficients, which the loss pass replaces row
  // by row with dL/dz (no dependent global load inside the pass)
  for (int r = rbeg + tid; r < rend; r += 64 * NW) bufA[r - rbeg] = cl[r];
  __syncthreads();
  {
    const FusedLossOp op{bufB, bufA, q, rbeg};
    stream_rows<FusedLossOp, 8>(g.went, g.wval, g.wrowid, op, mine.x, mine.y, lsum);
    for (int hh = h0; hh < h1; ++hh) {
      const int i = g.heavy_rows[hh];
      const float total = heavy_row_sum<FusedLossOp, 64 * NW>(g, g.ent, op, i, red);
      if (tid == 0) op.finish(i, total, lsum, op.row_inputs(i));
    }
  }
  lsum = wave_sum(lsum);
  if (lane == 0) dred[wave] = lsum;
  __syncthreads();  // also: dL/dz of every row is in bufA
  if (tid == 0) {
    double total = 0.0;
    for (int w = 0; w < NW; ++w) total += dred[w];
    loss_partial[k] = total;
  }
  if (passes < 3) return;
  {
    const FusedBackOp op{bufA, g_t, rbeg};
    stream_rows<FusedBackOp, 8>(g.went_t, g.wval_t, g.wrowid, op, mine.x, mine.y, lsum);
    for (int hh = h0; hh < h1; ++hh) {
      const int i = g.heavy_rows[hh];
      const float total = heavy_row_sum<FusedBackOp, 64 * NW>(g, g.ent_t, op, i, red);
      if (tid == 0) op.finish(i, total, lsum, op.row_inputs(i));
    }
  }
}

// ---------------------------------------------------------------------------
// One width-1 pass with the gathered vector of the subgraph in LDS: several workgroups of
// NW wavefronts per subgraph (ScalarStaging); each copies the subgraph's rows of the vector
// the pass gathers from (t, p or dL/dz) into LDS, then its wavefronts sum their ranges of
// the light stream with gathers that never leave the compute unit.  A
// gather of 64 scattered 4-byte values from memory costs the L1 one cache line per lane;
// from LDS it is one pass over the banks.  Rows with very many neighbours of subgraph k
// are dealt to its workgroups in turn.  loss_partial (LossOp) gets one value per workgroup.
// ---------------------------------------------------------------------------
template <class Op>
struct StagedOp {
  static constexpr bool kWeighted = Op::kWeighted;
  Op op;
  const float* buf;  // buf[i] = op.source()[base + i]
  int base;
  __device__ __forceinline__ float gather(int j) const { return buf[j - base]; }
  static constexpr bool kRowInputs = Op::kRowInputs;
  __device__ __forceinline__ float2 row_inputs(int i) const { return op.row_inputs(i); }
  __device__ __forceinline__ void finish(int i, float s, double& ls, float2 y) const { op.finish(i, s, ls, y); }
};

constexpr int kStagedLoads = 10;  // 16-byte loads per thread of the copy into LDS

template <class Op, int NW>
__global__ __launch_bounds__(64 * NW) void narrow_staged_kernel(GraphView g, Op op, ScalarStaging sg,
                                                                double* __restrict__ loss_partial) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* buf = reinterpret_cast<float*>(smem);
  float* red = buf + sg.cap;
  double* dred = reinterpret_cast<double*>(red + NW + (NW % 2));
  const int wg = sg.launch_of[blockIdx.x];
  if (wg < 0) return;
  const int k = sg.wg_k[wg];
  if (g.loss_ptr[k + 1] == g.loss_ptr[k]) return;  // the subgraph sits out
  const int s = wg - sg.wg_ptr[k], per = sg.wg_ptr[k + 1] - sg.wg_ptr[k];
  const int tid = threadIdx.x, lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int rbeg = g.part_rows[k], rend = g.part_rows[k + 1];
  const int2 mine = sg.cuts[static_cast<size_t>(wg) * NW + wave];
  const float* __restrict__ src = op.source();
  // The subgraph's rows of the gathered vector, from the 16-byte boundary at or before the
  // first one: buf[i] = src[abeg + i].  All loads of the copy are issued at once, before the
  // wavefront's first stream entries are requested (those take longer and vector memory
  // operations complete in order); the values go to LDS while the entries travel.
  const int abeg = rbeg & ~3;
  float4 staged[kStagedLoads];
#pragma unroll
  for (int u = 0; u < kStagedLoads; ++u) {
    const int idx = abeg + 4 * (tid + u * 64 * NW);
    staged[u] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (idx < rend) {
      if (idx + 3 < g.n) {
        staged[u] = *reinterpret_cast<const float4*>(src + idx);
      } else {  // the last rows of the whole vector
        staged[u].x = src[idx];
        if (idx + 1 < g.n) staged[u].y = src[idx + 1];
        if (idx + 2 < g.n) staged[u].z = src[idx + 2];
      }
    }
  }
  const StagedOp<Op> sop{op, buf, abeg};
  double lsum = 0.0;
  auto park = [&]() {
#pragma unroll
    for (int u = 0; u < kStagedLoads; ++u) {
      const int i4 = 4 * (tid + u * 64 * NW);
      if (abeg + i4 < rend) *reinterpret_cast<float4*>(buf + i4) = staged[u];
    }
    __syncthreads();
  };
  stream_rows<StagedOp<Op>, 4>(g.went, g.wval, g.wrowid, sop, mine.x, mine.y, lsum, park);
  for (int hh = sg.heavy_ptr[k] + s; hh < sg.heavy_ptr[k + 1]; hh += per) {
    const int i = g.heavy_rows[hh];
    const float total = heavy_row_sum<StagedOp<Op>, 64 * NW>(g, g.ent, sop, i, red);
    if (tid == 0) sop.finish(i, total, lsum, sop.row_inputs(i));
  }
  if (loss_partial != nullptr) {
    lsum = wave_sum(lsum);
    if (lane == 0) dred[wave] = lsum;
    __syncthreads();
    if (tid == 0) {
      double total = 0.0;
      for (int w = 0; w < NW; ++w) total += dred[w];
      loss_partial[wg] = total;
    }
  }
}

constexpr int kStagedWaves = 8;

template <class Op>
void launch_staged(const Launch& ln, int kind, const GraphView& g, const Op& op, const ScalarStaging& sg,
                   double* loss_partial) {
  const size_t lds = scalar_staged_lds_bytes(sg.cap);
  ln.begin(kind);
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(narrow_staged_kernel<Op, kStagedWaves>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
  narrow_staged_kernel<Op, kStagedWaves><<<sg.num_launch, 64 * kStagedWaves, lds, ln.st>>>(g, op, sg, loss_partial);
  ln.end(kind);
}

template <class Op>
void launch_narrow(const Launch& ln, int kind, const GraphView& g, const Op& op, double* loss_partial) {
  ln.begin(kind);
  narrow_stream_kernel<Op><<<g.num_hparts + g.num_wblocks[WM_NARROW], kBlock, 0, ln.st>>>(g, op, loss_partial);
  ln.end(kind);
}

}  // namespace

size_t scalar_fused_lds_bytes(int waves, int cap) {
  return 2 * static_cast<size_t>(cap) * sizeof(float) + static_cast<size_t>(waves + waves % 2) * sizeof(float) +
         static_cast<size_t>(waves) * sizeof(double);
}

void launch_scalar_fused(const Launch& ln, const GraphView& g, int waves, int cap, const int2* cuts,
                         const int* heavy_ptr, const float* t, float* p, const float* c, float q, float* g_t,
                         double* loss_partial, int passes) {
  const size_t lds = scalar_fused_lds_bytes(waves, cap);
  ln.begin(KK_SCALAR_FUSED);
  if (waves == 16) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(scalar_layer_fused_kernel<16>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    scalar_layer_fused_kernel<16><<<g.P, 1024, lds, ln.st>>>(g, cuts, heavy_ptr, cap, t, p, c, q, g_t,
                                                            loss_partial, passes);
  } else {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(scalar_layer_fused_kernel<4>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    scalar_layer_fused_kernel<4><<<g.P, 256, lds, ln.st>>>(g, cuts, heavy_ptr, cap, t, p, c, q, g_t,
                                                          loss_partial, passes);
  }
  ln.end(KK_SCALAR_FUSED);
}

int scalar_staged_waves() { return kStagedWaves; }
int scalar_staged_max_cap() { return 64 * kStagedWaves * 4 * kStagedLoads; }

size_t scalar_staged_lds_bytes(int cap) {
  return static_cast<size_t>(cap) * sizeof(float) + static_cast<size_t>(kStagedWaves) * (sizeof(float) + sizeof(double));
}

void launch_fwd_readout(const Launch& ln, const GraphView& g, const float* t, float* z, float* p,
                        const ScalarStaging* sg) {
  if (sg != nullptr) launch_staged(ln, KK_FWD_READOUT, g, ReadoutOp{t, z, p}, *sg, nullptr);
  else launch_narrow(ln, KK_FWD_READOUT, g, ReadoutOp{t, z, p}, nullptr);
}

void launch_loss(const Launch& ln, const GraphView& g, const float* p, const float* c, float q, float* g_z,
                 double* loss_partial, const ScalarStaging* sg) {
  if (sg != nullptr) launch_staged(ln, KK_LOSS, g, LossOp{p, c, q, g_z}, *sg, loss_partial);
  else launch_narrow(ln, KK_LOSS, g, LossOp{p, c, q, g_z}, loss_partial);
}

void launch_bwd_readout(const Launch& ln, const GraphView& g, const float* g_z, float* g_t,
                        const ScalarStaging* sg) {
  if (sg != nullptr) launch_staged(ln, KK_BWD_READOUT, transposed(g), BackOp{g_z, g_t}, *sg, nullptr);
  else launch_narrow(ln, KK_BWD_READOUT, transposed(g), BackOp{g_z, g_t}, nullptr);
}

}  // namespace gco
