// Integer kernels: graph checks and preprocessing at upload, cross-edge export,
// binarisation and greedy repair.  Everything here is exact.
#include "device_utils.h"
#include "graph_kernels.h"

namespace gco {
namespace {

// ---------------------------------------------------------------------------
// Exclusive prefix sum over int64 (three-phase, recursive on the block totals)
// ---------------------------------------------------------------------------
constexpr int kScanItems = 4;
constexpr int kScanTile = kBlock * kScanItems;

__global__ __launch_bounds__(kBlock) void scan_tiles_kernel(const int64_t* __restrict__ in,
                                                            int64_t* __restrict__ out, int64_t n,
                                                            int64_t* __restrict__ tile_sums) {
  __shared__ int64_t sh[kBlock];
  const int64_t base = static_cast<int64_t>(blockIdx.x) * kScanTile + threadIdx.x * kScanItems;
  int64_t v[kScanItems];
  int64_t sum = 0;
#pragma unroll
  for (int q = 0; q < kScanItems; ++q) {
    v[q] = (base + q < n) ? in[base + q] : 0;
    sum += v[q];
  }
  sh[threadIdx.x] = sum;
  __syncthreads();
  for (int off = 1; off < kBlock; off <<= 1) {
    const int64_t add = threadIdx.x >= off ? sh[threadIdx.x - off] : 0;
    __syncthreads();
    sh[threadIdx.x] += add;
    __syncthreads();
  }
  int64_t run = sh[threadIdx.x] - sum;  // exclusive prefix of this thread within the tile
#pragma unroll
  for (int q = 0; q < kScanItems; ++q) {
    if (base + q < n) out[base + q] = run;
    run += v[q];
  }
  if (threadIdx.x == kBlock - 1) tile_sums[blockIdx.x] = sh[kBlock - 1];
}

__global__ __launch_bounds__(kBlock) void scan_add_kernel(int64_t* __restrict__ out, int64_t n,
                                                          const int64_t* __restrict__ tile_offsets) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kScanTile + threadIdx.x;
  const int64_t off = tile_offsets[blockIdx.x];
#pragma unroll
  for (int q = 0; q < kScanItems; ++q) {
    const int64_t idx = i + static_cast<int64_t>(q) * kBlock;
    if (idx < n) out[idx] += off;
  }
}

}  // namespace

size_t scan_temp_elems(int64_t n) {
  size_t total = 0;
  while (n > 1) {
    n = (n + kScanTile - 1) / kScanTile;
    total += static_cast<size_t>(n) * 2;
    if (n == 1) break;
  }
  return total + 2;
}

// out[i] = sum_{j < i} in[i] for i in [0, n]; out has n + 1 entries (out[n] = total).
// `in` must have n + 1 readable entries with in[n] ignored (treated as 0 by
// passing n + 1 items whose last is overwritten by the caller with 0).
void exclusive_scan_i64(hipStream_t st, const int64_t* in, int64_t* out, int64_t count,
                        int64_t* temp) {
  if (count <= 0) return;
  const int64_t tiles = (count + kScanTile - 1) / kScanTile;
  int64_t* sums = temp;
  int64_t* sums_scanned = temp + tiles;
  scan_tiles_kernel<<<static_cast<unsigned>(tiles), kBlock, 0, st>>>(in, out, count, sums);
  if (tiles > 1) {
    exclusive_scan_i64(st, sums, sums_scanned, tiles, temp + 2 * tiles);
    scan_add_kernel<<<static_cast<unsigned>(tiles), kBlock, 0, st>>>(out, count, sums_scanned);
  }
}

namespace {

// ---------------------------------------------------------------------------
// Upload: checks
// ---------------------------------------------------------------------------
__device__ __forceinline__ int64_t row_of_entry(const int64_t* __restrict__ rowptr, int64_t n,
                                                int64_t e) {
  int64_t lo = 0, hi = n;  // last i with rowptr[i] <= e
  while (hi - lo > 1) {
    const int64_t mid = (lo + hi) >> 1;
    if (rowptr[mid] <= e) lo = mid; else hi = mid;
  }
  return lo;
}

// err[0] receives the largest code seen: 1 column out of range, 2 self loop,
// 3 columns not strictly ascending, 4 missing reverse entry.
__global__ __launch_bounds__(kBlock) void check_graph_kernel(int64_t n, const int64_t* __restrict__ rowptr,
                                                             const int32_t* __restrict__ col,
                                                             int64_t nnz, int* __restrict__ err) {
  const int64_t e = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (e >= nnz) return;
  const int64_t i = row_of_entry(rowptr, n, e);
  const int64_t j = col[e];
  int code = 0;
  if (j < 0 || j >= n) {
    code = 1;
  } else if (j == i) {
    code = 2;
  } else if (e > rowptr[i] && col[e - 1] >= j) {
    code = 3;
  } else {
    int64_t lo = rowptr[j], hi = rowptr[j + 1];  // find i in row j
    bool found = false;
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      const int32_t cv = col[mid];
      if (cv == i) { found = true; break; }
      if (cv < i) lo = mid + 1; else hi = mid;
    }
    if (!found) code = 4;
  }
  if (code) atomicMax(err, code);
}

// ---------------------------------------------------------------------------
// Upload: local CSR in subgraph-contiguous order
// ---------------------------------------------------------------------------
// One wavefront per new row r (original node perm[r]).
__global__ __launch_bounds__(kBlock) void local_count_kernel(int n, const int64_t* __restrict__ rowptr,
                                                             const int32_t* __restrict__ col,
                                                             const int32_t* __restrict__ part,
                                                             const int32_t* __restrict__ perm,
                                                             int64_t* __restrict__ count) {
  const int r = blockIdx.x * (kBlock / 64) + threadIdx.x / 64;
  if (r >= n) return;
  const int lane = threadIdx.x % 64;
  const int i = perm[r];
  const int pk = part[i];
  int c = 0;
  for (int64_t e = rowptr[i] + lane; e < rowptr[i + 1]; e += 64) c += (part[col[e]] == pk) ? 1 : 0;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off, 64);
  if (lane == 0) count[r] = c;
}

__global__ __launch_bounds__(kBlock) void local_fill_kernel(int n, const int64_t* __restrict__ rowptr,
                                                            const int32_t* __restrict__ col,
                                                            const int32_t* __restrict__ part,
                                                            const int32_t* __restrict__ perm,
                                                            const int32_t* __restrict__ inv,
                                                            const int64_t* __restrict__ lptr64,
                                                            int32_t* __restrict__ lrowptr,
                                                            int32_t* __restrict__ lcol) {
  const int r = blockIdx.x * (kBlock / 64) + threadIdx.x / 64;
  if (r > n) return;
  const int lane = threadIdx.x % 64;
  if (r == n) {
    if (lane == 0) lrowptr[n] = static_cast<int32_t>(lptr64[n]);
    return;
  }
  const int i = perm[r];
  const int pk = part[i];
  int64_t outp = lptr64[r];
  if (lane == 0) lrowptr[r] = static_cast<int32_t>(outp);
  const int64_t e0 = rowptr[i], e1 = rowptr[i + 1];
  for (int64_t eb = e0; eb < e1; eb += 64) {
    const int64_t e = eb + lane;
    int j = -1;
    bool keep = false;
    if (e < e1) {
      j = col[e];
      keep = part[j] == pk;
    }
    const unsigned long long mask = __ballot(keep);
    if (keep) {
      const int before = __popcll(mask & ((1ull << lane) - 1ull));
      lcol[outp + before] = inv[j];
    }
    outp += __popcll(mask);
  }
}

// sa, sb (A_hat_ij = sa_i * sb_j), the local degree and the linear coefficient.
__global__ __launch_bounds__(kBlock) void scales_kernel(int n, const int32_t* __restrict__ lrowptr,
                                                        int norm, int problem, float beta,
                                                        float* __restrict__ sa, float* __restrict__ sb,
                                                        float* __restrict__ c_base) {
  const int r = blockIdx.x * kBlock + threadIdx.x;
  if (r >= n) return;
  const int deg = lrowptr[r + 1] - lrowptr[r];
  const double dt = static_cast<double>(deg) + 1.0;
  if (norm == GCO_NORM_MEAN) {
    sa[r] = static_cast<float>(1.0 / dt);
    sb[r] = 1.f;
  } else {
    const float s = static_cast<float>(1.0 / sqrt(dt));
    sa[r] = s;
    sb[r] = s;
  }
  c_base[r] = problem == GCO_PROBLEM_MAXCUT ? -static_cast<float>(deg) : -beta;
}

// One wavefront per row i: ent[e] = {j, row_scale[i] * col_scale[j]} for its entries
// e = (i, j); with diag != nullptr also diag[i] = row_scale[i] * col_scale[i].
__global__ __launch_bounds__(kBlock) void pack_entries_kernel(int n, const int32_t* __restrict__ rowptr,
                                                              const int32_t* __restrict__ col,
                                                              const float* __restrict__ row_scale,
                                                              const float* __restrict__ col_scale,
                                                              int2* __restrict__ ent,
                                                              float* __restrict__ diag) {
  const int i = blockIdx.x * (kBlock / 64) + threadIdx.x / 64;
  if (i >= n) return;
  const int lane = threadIdx.x % 64;
  const float ri = row_scale[i];
  if (diag != nullptr && lane == 0) diag[i] = ri * col_scale[i];
  for (int e = rowptr[i] + lane; e < rowptr[i + 1]; e += 64) {
    const int j = col[e];
    ent[e] = make_int2(j, __float_as_int(ri * col_scale[j]));
  }
}

// count[i] = number of entries of row i in the light stream: its diagonal entry, and
// its neighbours unless the row is pre-reduced
__global__ __launch_bounds__(kBlock) void light_count_kernel(int n, const int32_t* __restrict__ rowptr,
                                                             int64_t* __restrict__ count) {
  const int i = blockIdx.x * kBlock + threadIdx.x;
  if (i >= n) return;
  const int deg = rowptr[i + 1] - rowptr[i];
  count[i] = 1 + (deg >= kHeavyMin ? 0 : deg);
}

// An fp32 value as two bf16 numbers hi + lo (hi in the upper half of the word): hi is the
// value rounded to bf16, lo the rounded remainder.
__device__ __forceinline__ int split_bf16(float w) {
  const uint32_t hi = f32_to_bf16(w);
  const uint32_t lo = f32_to_bf16(w - __uint_as_float(hi << 16));
  return static_cast<int>((hi << 16) | lo);
}

// One wavefront per row: {i, diag[i]}, then a light row's entries, to the light stream,
// the values split into bf16 pairs.  wrowid (may be null) receives the row of every entry of
// the stream, -2 for the lone entry of a pre-reduced row.
__global__ __launch_bounds__(kBlock) void light_fill_kernel(int n, const int32_t* __restrict__ rowptr,
                                                            const int2* __restrict__ ent,
                                                            const float* __restrict__ diag,
                                                            const int64_t* __restrict__ wptr64,
                                                            int32_t* __restrict__ wrowptr,
                                                            int2* __restrict__ went,
                                                            float* __restrict__ wval,
                                                            int32_t* __restrict__ wrowid) {
  const int i = blockIdx.x * (kBlock / 64) + threadIdx.x / 64;
  if (i > n) return;
  const int lane = threadIdx.x % 64;
  if (lane == 0) wrowptr[i] = static_cast<int32_t>(wptr64[i]);
  if (i == n) return;
  const int64_t out = wptr64[i];
  const int deg = rowptr[i + 1] - rowptr[i];
  if (lane == 0) {
    went[out] = make_int2(i, split_bf16(diag[i]));
    wval[out] = diag[i];
    if (wrowid != nullptr) wrowid[out] = deg >= kHeavyMin ? -2 : i;
  }
  if (deg >= kHeavyMin) return;
  for (int q = lane; q < deg; q += 64) {
    const int2 en = ent[rowptr[i] + q];
    went[out + 1 + q] = make_int2(en.x, split_bf16(__int_as_float(en.y)));
    wval[out + 1 + q] = __int_as_float(en.y);
    if (wrowid != nullptr) wrowid[out + 1 + q] = i;
  }
}

// c[r] = c_base[r] + extra_orig[perm[r]]
__global__ __launch_bounds__(kBlock) void linear_coeff_kernel(int n, const float* __restrict__ c_base,
                                                              const float* __restrict__ extra_orig,
                                                              const int32_t* __restrict__ perm,
                                                              float* __restrict__ c) {
  const int r = blockIdx.x * kBlock + threadIdx.x;
  if (r >= n) return;
  c[r] = c_base[r] + (extra_orig ? extra_orig[perm[r]] : 0.f);
}

// ---------------------------------------------------------------------------
// Row permutations between original and subgraph-contiguous order
// ---------------------------------------------------------------------------
// dst[r, :] = src[map[r], :]  (width elements of 4 bytes per row)
__global__ __launch_bounds__(kBlock) void gather_rows_kernel(int64_t total, int width,
                                                             const uint32_t* __restrict__ src,
                                                             const int32_t* __restrict__ map,
                                                             uint32_t* __restrict__ dst) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (idx >= total) return;
  const int64_t r = idx / width;
  const int c = static_cast<int>(idx % width);
  dst[idx] = src[static_cast<int64_t>(map[r]) * width + c];
}

__global__ __launch_bounds__(kBlock) void gather_bytes_kernel(int n, const uint8_t* __restrict__ src,
                                                              const int32_t* __restrict__ map,
                                                              uint8_t* __restrict__ dst) {
  const int i = blockIdx.x * kBlock + threadIdx.x;
  if (i < n) dst[i] = src[map[i]];
}

// ---------------------------------------------------------------------------
// Cross edges
// ---------------------------------------------------------------------------
// One wavefront per original row: entries (i, j) with j > i and part differs
// (optionally also x[i] = x[j] = 1).
__global__ __launch_bounds__(kBlock) void cut_count_kernel(int n, const int64_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ col,
                                                           const int32_t* __restrict__ part,
                                                           const uint8_t* __restrict__ x,
                                                           int64_t* __restrict__ count) {
  const int i = blockIdx.x * (kBlock / 64) + threadIdx.x / 64;
  if (i >= n) return;
  const int lane = threadIdx.x % 64;
  const int pk = part[i];
  int c = 0;
  if (x == nullptr || x[i]) {
    for (int64_t e = rowptr[i] + lane; e < rowptr[i + 1]; e += 64) {
      const int j = col[e];
      c += (j > i && part[j] != pk && (x == nullptr || x[j])) ? 1 : 0;
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off, 64);
  if (lane == 0) count[i] = c;
}

__global__ __launch_bounds__(kBlock) void cut_fill_kernel(int n, const int64_t* __restrict__ rowptr,
                                                          const int32_t* __restrict__ col,
                                                          const int32_t* __restrict__ part,
                                                          const uint8_t* __restrict__ x,
                                                          const int64_t* __restrict__ offs,
                                                          int32_t* __restrict__ u, int32_t* __restrict__ v,
                                                          uint8_t* __restrict__ cross) {
  const int i = blockIdx.x * (kBlock / 64) + threadIdx.x / 64;
  if (i >= n) return;
  const int lane = threadIdx.x % 64;
  if (x != nullptr && !x[i]) return;
  const int pk = part[i];
  int64_t outp = offs[i];
  const int64_t e0 = rowptr[i], e1 = rowptr[i + 1];
  for (int64_t eb = e0; eb < e1; eb += 64) {
    const int64_t e = eb + lane;
    int j = -1;
    bool keep = false;
    if (e < e1) {
      j = col[e];
      keep = j > i && part[j] != pk && (x == nullptr || x[j]);
    }
    const unsigned long long mask = __ballot(keep);
    if (keep) {
      const int64_t pos = outp + __popcll(mask & ((1ull << lane) - 1ull));
      if (u) { u[pos] = i; v[pos] = j; }
      if (cross) { cross[i] = 1; cross[j] = 1; }
    }
    outp += __popcll(mask);
  }
}

// ---------------------------------------------------------------------------
// Binarisation, greedy repair, counts
// ---------------------------------------------------------------------------
// state: 0 = not selected or removed, 1 = selected and undecided, 2 = kept
__global__ __launch_bounds__(kBlock) void round_kernel(int n, const float* __restrict__ p, float thr,
                                                       uint8_t* __restrict__ state) {
  const int i = blockIdx.x * kBlock + threadIdx.x;
  if (i < n) state[i] = p[i] >= thr ? 1 : 0;
}

// One wavefront per undecided node.  A node is removed once a kept neighbour
// of higher priority exists, kept once every selected neighbour of higher
// priority has been removed.  Priority: p descending, then index ascending.
// States only move 1 -> 0 or 1 -> 2 and every decision rests on final facts,
// so the fixed point does not depend on the interleaving.
template <typename PtrT>
__global__ __launch_bounds__(kBlock) void repair_round_kernel(int n, const PtrT* __restrict__ rowptr,
                                                              const int32_t* __restrict__ col,
                                                              const int32_t* __restrict__ part,
                                                              const float* __restrict__ p,
                                                              volatile uint8_t* state,
                                                              int* __restrict__ undecided) {
  const int i = blockIdx.x * (kBlock / 64) + threadIdx.x / 64;
  if (i >= n) return;
  if (state[i] != 1) return;
  const int lane = threadIdx.x % 64;
  const float pi = p[i];
  const int pk = part ? part[i] : 0;
  bool kill = false, wait = false;
  for (PtrT eb = rowptr[i]; eb < rowptr[i + 1]; eb += 64) {
    const PtrT e = eb + lane;
    if (e < rowptr[i + 1]) {
      const int j = col[e];
      if (part == nullptr || part[j] == pk) {
        const uint8_t sj = state[j];
        if (sj != 0) {
          const float pj = p[j];
          if (pj > pi || (pj == pi && j < i)) {
            if (sj == 2) kill = true; else wait = true;
          }
        }
      }
    }
    if (__ballot(kill)) break;
  }
  const bool any_kill = __ballot(kill) != 0ull;
  const bool any_wait = __ballot(wait) != 0ull;
  if (lane == 0) {
    if (any_kill) state[i] = 0;
    else if (!any_wait) state[i] = 2;
    else atomicAdd(undecided, 1);
  }
}

__global__ __launch_bounds__(kBlock) void state_to_x_kernel(int n, const uint8_t* __restrict__ state,
                                                            uint8_t* __restrict__ x) {
  const int i = blockIdx.x * kBlock + threadIdx.x;
  if (i < n) x[i] = state[i] != 0 ? 1 : 0;
}

// counts[0] += |{i: x_i = 1}|, counts[1] += edges with both ends 1,
// counts[2] += edges whose ends differ (each undirected edge once, i < j).
__global__ __launch_bounds__(kBlock) void edge_counts_kernel(int n, const int64_t* __restrict__ rowptr,
                                                             const int32_t* __restrict__ col,
                                                             const uint8_t* __restrict__ x,
                                                             unsigned long long* __restrict__ counts) {
  // one wavefront per row, 16 rows per wavefront; integer sums are combined per
  // workgroup before the three atomics, so the totals are exact and contention is low
  __shared__ unsigned int part[3][kBlock / 64];
  const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
  unsigned int sel = 0, both = 0, differ = 0;
  for (int q = 0; q < 16; ++q) {
    const int i = (blockIdx.x * 16 + q) * (kBlock / 64) + wave;
    if (i >= n) break;
    const int xi = x[i];
    if (lane == 0) sel += xi;
    for (int64_t e = rowptr[i] + lane; e < rowptr[i + 1]; e += 64) {
      const int j = col[e];
      if (j > i) {
        const int xj = x[j];
        both += (xi & xj);
        differ += (xi ^ xj);
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    sel += __shfl_xor(sel, off, 64);
    both += __shfl_xor(both, off, 64);
    differ += __shfl_xor(differ, off, 64);
  }
  if (lane == 0) {
    part[0][wave] = sel;
    part[1][wave] = both;
    part[2][wave] = differ;
  }
  __syncthreads();
  if (threadIdx.x < 3) {
    unsigned long long tot = 0;
    for (int w = 0; w < kBlock / 64; ++w) tot += part[threadIdx.x][w];
    if (tot) atomicAdd(&counts[threadIdx.x], tot);
  }
}

__global__ __launch_bounds__(kBlock) void fill_u32_kernel(uint32_t* __restrict__ dst, int64_t count,
                                                          uint32_t value) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (i < count) dst[i] = value;
}

inline unsigned blocks_for(int64_t items, int per_block) {
  return static_cast<unsigned>((items + per_block - 1) / per_block);
}

}  // namespace

void launch_check_graph(hipStream_t st, int64_t n, const int64_t* rowptr, const int32_t* col,
                        int64_t nnz, int* err) {
  if (nnz > 0) check_graph_kernel<<<blocks_for(nnz, kBlock), kBlock, 0, st>>>(n, rowptr, col, nnz, err);
}

void launch_local_count(hipStream_t st, int n, const int64_t* rowptr, const int32_t* col,
                        const int32_t* part, const int32_t* perm, int64_t* count) {
  local_count_kernel<<<blocks_for(n, kBlock / 64), kBlock, 0, st>>>(n, rowptr, col, part, perm, count);
}

void launch_local_fill(hipStream_t st, int n, const int64_t* rowptr, const int32_t* col,
                       const int32_t* part, const int32_t* perm, const int32_t* inv,
                       const int64_t* lptr64, int32_t* lrowptr, int32_t* lcol) {
  local_fill_kernel<<<blocks_for(static_cast<int64_t>(n) + 1, kBlock / 64), kBlock, 0, st>>>(
      n, rowptr, col, part, perm, inv, lptr64, lrowptr, lcol);
}

void launch_scales(hipStream_t st, int n, const int32_t* lrowptr, int norm, int problem, float beta,
                   float* sa, float* sb, float* c_base) {
  scales_kernel<<<blocks_for(n, kBlock), kBlock, 0, st>>>(n, lrowptr, norm, problem, beta, sa, sb, c_base);
}

void launch_pack_entries(hipStream_t st, int n, const int32_t* rowptr, const int32_t* col,
                         const float* row_scale, const float* col_scale, int2* ent, float* diag) {
  pack_entries_kernel<<<blocks_for(n, kBlock / 64), kBlock, 0, st>>>(n, rowptr, col, row_scale, col_scale,
                                                                      ent, diag);
}

void launch_light_count(hipStream_t st, int n, const int32_t* rowptr, int64_t* count) {
  light_count_kernel<<<blocks_for(n, kBlock), kBlock, 0, st>>>(n, rowptr, count);
}

void launch_light_fill(hipStream_t st, int n, const int32_t* rowptr, const int2* ent, const float* diag,
                       const int64_t* wptr64, int32_t* wrowptr, int2* went, float* wval, int32_t* wrowid) {
  light_fill_kernel<<<blocks_for(static_cast<int64_t>(n) + 1, kBlock / 64), kBlock, 0, st>>>(
      n, rowptr, ent, diag, wptr64, wrowptr, went, wval, wrowid);
}

void launch_linear_coeff(hipStream_t st, int n, const float* c_base, const float* extra_orig,
                         const int32_t* perm, float* c) {
  linear_coeff_kernel<<<blocks_for(n, kBlock), kBlock, 0, st>>>(n, c_base, extra_orig, perm, c);
}

void launch_gather_rows(hipStream_t st, int64_t rows, int width, const void* src, const int32_t* map,
                        void* dst) {
  const int64_t total = rows * width;
  if (total > 0)
    gather_rows_kernel<<<blocks_for(total, kBlock), kBlock, 0, st>>>(
        total, width, static_cast<const uint32_t*>(src), map, static_cast<uint32_t*>(dst));
}

void launch_gather_bytes(hipStream_t st, int n, const uint8_t* src, const int32_t* map, uint8_t* dst) {
  gather_bytes_kernel<<<blocks_for(n, kBlock), kBlock, 0, st>>>(n, src, map, dst);
}

void launch_cut_count(hipStream_t st, int n, const int64_t* rowptr, const int32_t* col,
                      const int32_t* part, const uint8_t* x, int64_t* count) {
  cut_count_kernel<<<blocks_for(n, kBlock / 64), kBlock, 0, st>>>(n, rowptr, col, part, x, count);
}

void launch_cut_fill(hipStream_t st, int n, const int64_t* rowptr, const int32_t* col,
                     const int32_t* part, const uint8_t* x, const int64_t* offs, int32_t* u,
                     int32_t* v, uint8_t* cross) {
  cut_fill_kernel<<<blocks_for(n, kBlock / 64), kBlock, 0, st>>>(n, rowptr, col, part, x, offs, u, v, cross);
}

void launch_round(hipStream_t st, int n, const float* p, float thr, uint8_t* state) {
  round_kernel<<<blocks_for(n, kBlock), kBlock, 0, st>>>(n, p, thr, state);
}

void launch_repair_round_local(hipStream_t st, int n, const int32_t* lrowptr, const int32_t* lcol,
                               const float* p, uint8_t* state, int* undecided) {
  repair_round_kernel<int32_t><<<blocks_for(n, kBlock / 64), kBlock, 0, st>>>(
      n, lrowptr, lcol, nullptr, p, state, undecided);
}

void launch_repair_round_all(hipStream_t st, int n, const int64_t* rowptr, const int32_t* col,
                             const float* p, uint8_t* state, int* undecided) {
  repair_round_kernel<int64_t><<<blocks_for(n, kBlock / 64), kBlock, 0, st>>>(
      n, rowptr, col, nullptr, p, state, undecided);
}

void launch_state_to_x(hipStream_t st, int n, const uint8_t* state, uint8_t* x) {
  state_to_x_kernel<<<blocks_for(n, kBlock), kBlock, 0, st>>>(n, state, x);
}

void launch_edge_counts(hipStream_t st, int n, const int64_t* rowptr, const int32_t* col,
                        const uint8_t* x, unsigned long long* counts) {
  edge_counts_kernel<<<blocks_for(n, 16 * (kBlock / 64)), kBlock, 0, st>>>(n, rowptr, col, x, counts);
}

void launch_fill_u32(hipStream_t st, void* dst, int64_t count, uint32_t value) {
  if (count > 0)
    fill_u32_kernel<<<blocks_for(count, kBlock), kBlock, 0, st>>>(static_cast<uint32_t*>(dst), count, value);
}

}  // namespace gco
