// Launchers of the integer kernels (graph_kernels.hip).  All pointers are device
// pointers; every launch is asynchronous on the given stream.
#pragma once

#include "gco_internal.h"

namespace gco {

// Exclusive prefix sum of `count` int64 items (out[i] = sum of in[0..i)).
// temp needs scan_temp_elems(count) int64 entries.
size_t scan_temp_elems(int64_t count);
void exclusive_scan_i64(hipStream_t st, const int64_t* in, int64_t* out, int64_t count,
                        int64_t* temp);

// err[0] = max over entries of: 1 column out of range, 2 self loop, 3 columns of
// a row not strictly ascending, 4 reverse entry missing.  rowptr must already
// be known to be monotone with rowptr[0] = 0, rowptr[n] = nnz.
void launch_check_graph(hipStream_t st, int64_t n, const int64_t* rowptr, const int32_t* col,
                        int64_t nnz, int* err);

// Local (same-subgraph) entries per row of the new order; then the local CSR.
void launch_local_count(hipStream_t st, int n, const int64_t* rowptr, const int32_t* col,
                        const int32_t* part, const int32_t* perm, int64_t* count);
void launch_local_fill(hipStream_t st, int n, const int64_t* rowptr, const int32_t* col,
                       const int32_t* part, const int32_t* perm, const int32_t* inv,
                       const int64_t* lptr64, int32_t* lrowptr, int32_t* lcol);
void launch_scales(hipStream_t st, int n, const int32_t* lrowptr, int norm, int problem, float beta,
                   float* sa, float* sb, float* c_base);
// ent[e] = {j, bits of row_scale[i] * col_scale[j]} for every local entry e = (i, j);
// diag[i] = row_scale[i] * col_scale[i] if diag is given.
void launch_pack_entries(hipStream_t st, int n, const int32_t* rowptr, const int32_t* col,
                         const float* row_scale, const float* col_scale, int2* ent, float* diag);
// Light stream (every row's diagonal entry {i, diag[i]}, followed by its entries unless the
// row is pre-reduced): per-row entry counts, then the fill at scanned offsets; went holds
// {column, value as a bf16 pair}, wval the value in fp32.
void launch_light_count(hipStream_t st, int n, const int32_t* rowptr, int64_t* count);
void launch_light_fill(hipStream_t st, int n, const int32_t* rowptr, const int2* ent, const float* diag,
                       const int64_t* wptr64, int32_t* wrowptr, int2* went, float* wval, int32_t* wrowid);
void launch_linear_coeff(hipStream_t st, int n, const float* c_base, const float* extra_orig,
                         const int32_t* perm, float* c);

// dst[r, :] = src[map[r], :] for rows of `width` 4-byte elements; and for bytes.
void launch_gather_rows(hipStream_t st, int64_t rows, int width, const void* src, const int32_t* map,
                        void* dst);
void launch_gather_bytes(hipStream_t st, int n, const uint8_t* src, const int32_t* map, uint8_t* dst);

// Cross edges: per-row counts, then the fill at scanned offsets.  x (optional)
// restricts to edges with both ends selected.  u, v, cross may each be nullptr.
void launch_cut_count(hipStream_t st, int n, const int64_t* rowptr, const int32_t* col,
                      const int32_t* part, const uint8_t* x, int64_t* count);
void launch_cut_fill(hipStream_t st, int n, const int64_t* rowptr, const int32_t* col,
                     const int32_t* part, const uint8_t* x, const int64_t* offs, int32_t* u,
                     int32_t* v, uint8_t* cross);

// Binarisation and one round of the parallel greedy repair (see the kernel).
void launch_round(hipStream_t st, int n, const float* p, float thr, uint8_t* state);
void launch_repair_round_local(hipStream_t st, int n, const int32_t* lrowptr, const int32_t* lcol,
                               const float* p, uint8_t* state, int* undecided);
void launch_repair_round_all(hipStream_t st, int n, const int64_t* rowptr, const int32_t* col,
                             const float* p, uint8_t* state, int* undecided);
void launch_state_to_x(hipStream_t st, int n, const uint8_t* state, uint8_t* x);
// counts[0] += selected nodes, counts[1] += edges with both ends selected,
// counts[2] += edges whose ends differ.
void launch_edge_counts(hipStream_t st, int n, const int64_t* rowptr, const int32_t* col,
                        const uint8_t* x, unsigned long long* counts);
void launch_fill_u32(hipStream_t st, void* dst, int64_t count, uint32_t value);

}  // namespace gco
