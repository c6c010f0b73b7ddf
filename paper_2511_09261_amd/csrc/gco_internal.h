// Internal declarations shared by the host API and the HIP kernel files.
// Nothing here is part of the public ABI (see include/gco.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "gco.h"

namespace gco {

constexpr int kBlock = 256;      // threads per workgroup in every kernel here (4 wavefronts)
constexpr int kTileRows = 64;    // rows of one feature tile in the wide kernels
constexpr int kNarrowRows = 256; // rows of one tile in the width-1 kernels
constexpr int kLightMax = 64;    // rows with more local neighbours are reduced by the whole block
constexpr int kHeavyMin = 256;   // rows with at least this many neighbours are pre-reduced in chunks
constexpr int kChunk = 256;      // neighbours per chunk of a pre-reduced row
constexpr int kNarrowPartChunks = 8;  // width-1 passes: chunks of a pre-reduced row summed by one workgroup
constexpr int kWideBlocks = 2048;        // workgroups aimed at by the wide kernels
constexpr int kMaxTilesPerBlock = 16;     // tiles one wide workgroup may own
constexpr int kWaveRows = 32;            // rows of a tile in the wave-per-tile kernels
// cuts of the tiles among the wavefronts, one per kernel kind: cost of a row relative to
// one light-stream entry (measured per-tile against per-entry time of each kernel)
enum WaveMap : int { WM_FWD = 0, WM_BWD = 1, WM_EMBED = 2, WM_NARROW = 3, WM_GRADW = 4, kWaveMaps = 5 };
constexpr double kWaveRowCost[kWaveMaps] = {1.25, 1.5, 100.0, 1.0, 100.0};
// workgroups aimed at (measured best); WM_GRADW: one per compute unit, which is all that fit at its size
constexpr int kWaveBlocksFor[kWaveMaps] = {768, 512, 3072, 2048, 256};
// width 128 (two workgroups of the layer kernels per compute unit): forward two rounds of 512,
// embedding backward twelve
constexpr int kWaveBlocksFor128[kWaveMaps] = {1024, 1024, 6144, 2048, 256};
constexpr int kEntPad = 512;             // zero entries appended to the packed entry arrays
// gco_round_repair_static works inside a block of device memory that is part of the
// library's code object: up to this many nodes, 7 bytes per node plus counters.
constexpr int kStaticMaxNodes = 1 << 21;
constexpr size_t kStaticScratchBytes = static_cast<size_t>(kStaticMaxNodes) * 7 + 4096;
hipError_t static_scratch_for_current_device(void** out);

constexpr int kMaxParts = 16384;         // subgraphs per graph (their loss sums share 128 KB of LDS)

enum KernelKind : int {
  KK_FWD_HIDDEN = 0,   // aggregate + transform + ReLU of one hidden layer (Eq. 3)
  KK_FWD_GEMV,         // t = E w (only when there is no hidden layer)
  KK_FWD_READOUT,      // z = A_hat t, p = sigmoid(z) (Eq. 4)
  KK_LOSS,             // loss and dL/dz (Eq. 5)
  KK_BWD_READOUT,      // g_t = A_hat^T g_z
  KK_BWD_HIDDEN,       // backward of a hidden layer that is not the first
  KK_BWD_EMBED,        // backward of the first layer + Adam on the embeddings
  KK_ADAM_W,           // gradient reduction + Adam on the weight matrices
  KK_LOSS_REDUCE,      // per-subgraph and total loss
  KK_HEAVY,            // chunked pre-reduction of very long rows
  KK_FORM_GZ,          // G_Z of the last hidden layer + gradient of the scalar layer's weights
  KK_BEST,             // best-by-loss snapshot: decision per model + copy of the improved ones
  KK_GRAD_W,           // weight gradient of a hidden layer from stored rows (bf16, width 128)
  KK_SCALAR_FUSED,     // read-out, loss and the scalar layer's backward aggregation in one launch
  KK_COUNT
};

// One wavefront's share of a wave-per-tile kernel.  Everything the wavefront needs before
// its first loads of the stream sits in this one 32-byte record, so that it starts them
// after a single lookup.
struct __attribute__((aligned(16))) WaveRun {
  int tile0, tile1;  // tiles [tile0, tile1) of its subgraph (kWaveRows rows each, from the subgraph's first row)
  int rbeg, rend;    // rows of the subgraph
  int e0, e1;        // light-stream range of the run's rows
  int tglob;         // global number of the subgraph's first tile
  int pad;
};

// Device view of the local (trained-on) graph in subgraph-contiguous node order,
// plus the static work decomposition.  All pointers are device pointers.
struct GraphView {
  int n = 0;
  int P = 0;
  const int* rowptr = nullptr;    // [n+1] local CSR
  const int* col = nullptr;       // [nnz]
  const float* sa = nullptr;      // [n] row scale of A_hat   (A_hat_ij = sa_i * sb_j)
  const float* sb = nullptr;      // [n] column scale of A_hat
  // the CSR entries again, packed as {column j, bits of A_hat_ij = sa_i sb_j};
  // ent_t carries A_hat_ji = sa_j sb_i instead (the entries of A_hat^T);
  // diag[i] = A_hat_ii = sa_i sb_i
  const int2* ent = nullptr;      // [nnz]
  const int2* ent_t = nullptr;    // [nnz]
  const float* diag = nullptr;    // [n]
  const int* part_rows = nullptr; // [P+1] first row of each subgraph
  // wide kernels: workgroup b works on tiles blk_s[b], + blk_S[b], + 2 blk_S[b], ...
  // of subgraph blk_k[b] (blk_k[b] < 0: nothing to do)
  const int* blk_k = nullptr;
  const int* blk_s = nullptr;
  const int* blk_S = nullptr;
  int num_blocks = 0;
  // wave-per-tile kernels, one decomposition per kernel kind m (WaveMap): workgroup b
  // serves subgraph wblk_k[m][b] (< 0: nothing to do); its wavefront q owns the tiles of
  // wave_runs[m][4b+q] -- contiguous runs, cut so that the wavefronts have about equal work
  // in that kind
  const int* wblk_k[kWaveMaps] = {};
  const WaveRun* wave_runs[kWaveMaps] = {};
  int num_wblocks[kWaveMaps] = {};
  // light stream: per row its diagonal entry {i, A_hat_ii}, then its packed entries unless
  // the row is pre-reduced; row i owns went[wrowptr[i] .. wrowptr[i+1]).  went_t holds the
  // entries of A_hat^T.  kEntPad zero entries follow the last row.
  const int* wrowptr = nullptr;   // [n+1]
  // wave tiles are numbered subgraph by subgraph: tile tau of subgraph k has the global
  // number (WaveRun::tglob of the subgraph) + tau; the pre-reduced rows inside global tile
  // T are heavy_rows[wtile_hptr[T] .. wtile_hptr[T+1])
  const int* wtile_hptr = nullptr;  // [tiles+1]
  const int2* went = nullptr;
  const int2* went_t = nullptr;
  // the same entries' values in fp32 (width-1 kernels), and the row every entry of the
  // stream belongs to (-2 for the lone entry of a pre-reduced row; the same for A_hat and
  // its transpose)
  const float* wval = nullptr;
  const float* wval_t = nullptr;
  const int* wrowid = nullptr;
  // narrow kernels: same scheme with kNarrowRows-row tiles
  const int* nblk_k = nullptr;
  const int* nblk_s = nullptr;
  const int* nblk_S = nullptr;
  int num_nblocks = 0;
  // loss partials: one per pre-reduced row (num_heavy), then one per workgroup of
  // decomposition WM_NARROW; those of subgraph k are loss_list[loss_ptr[k] .. loss_ptr[k+1])
  int num_loss_slots = 0;
  const int* loss_ptr = nullptr;
  const int* loss_list = nullptr;
  // very long rows, pre-reduced in chunks: row heavy_row[h] owns chunks
  // heavy_chunk_ptr[h] .. heavy_chunk_ptr[h+1]; chunk c covers CSR entries
  // chunk_begin[c] .. chunk_end[c].  heavy_of_row[i] = h or -1.
  int num_heavy = 0;
  int num_chunks = 0;
  const int* heavy_of_row = nullptr;  // [n]
  const int* heavy_rows = nullptr;    // [num_heavy] ascending row ids (< 0: a row of a subgraph that sits out)
  const int* heavy_chunk_ptr = nullptr;
  const int* chunk_begin = nullptr;
  const int* chunk_end = nullptr;
  const int* chunk_part = nullptr;    // subgraph of the row that owns the chunk (< 0: skip the chunk)
  // Width-1 passes as three launches: a pre-reduced row is summed by one workgroup per
  // kNarrowPartChunks of its chunks ("part").  hpart[q] = {h, index of the part in row h};
  // row h owns partial sums hpart_partial[hpart_ptr[h] .. hpart_ptr[h+1]); the workgroup that
  // finds hpart_count[h] at (parts - 1) adds them in order, applies the row's epilogue and
  // puts the count back to zero.
  int num_hparts = 0;
  const int2* hpart = nullptr;
  const int* hpart_ptr = nullptr;
  float* hpart_partial = nullptr;
  int* hpart_count = nullptr;
};

// The view of the transposed matrix: scale vectors and entry arrays exchanged.
inline GraphView transposed(const GraphView& g) {
  GraphView gt = g;
  gt.sa = g.sb;
  gt.sb = g.sa;
  gt.ent = g.ent_t;
  gt.ent_t = g.ent;
  gt.went = g.went_t;
  gt.went_t = g.went;
  gt.wval = g.wval_t;
  gt.wval_t = g.wval;
  return gt;
}

// Per-call Adam constants (bias corrections evaluated on the host in double).
struct AdamStep {
  float lr, b1, b2, eps;
  float inv_bc1;       // 1 / (1 - b1^t)
  float inv_sqrt_bc2;  // 1 / sqrt(1 - b2^t)
  // When the subgraphs (weight sets) have seen different numbers of steps: the two bias
  // corrections per subgraph, {inv_bc1, inv_sqrt_bc2}[k]; nullptr = the values above.
  const float2* per_part = nullptr;
  __host__ __device__ AdamStep for_part(int k) const {
    AdamStep r = *this;
#if defined(__HIP_DEVICE_COMPILE__)
    if (per_part != nullptr) {
      const float2 bc = per_part[k];
      r.inv_bc1 = bc.x;
      r.inv_sqrt_bc2 = bc.y;
    }
#else
    (void)k;
#endif
    return r;
  }
};

// Where to enqueue, and an optional per-kernel timer: begin/end bracket exactly
// one kernel launch of the given kind with events on the stream.
struct Profiler {
  virtual void begin(int kind, hipStream_t st) = 0;
  virtual void end(int kind, hipStream_t st) = 0;
  virtual ~Profiler() {}
};
struct Launch {
  hipStream_t st = nullptr;
  Profiler* prof = nullptr;
  void begin(int kind) const { if (prof) prof->begin(kind, st); }
  void end(int kind) const { if (prof) prof->end(kind, st); }
};

enum EmbedMode : int { EMBED_ADAM = 0, EMBED_WRITE_GRAD = 1, EMBED_SKIP = 2 };

// ---- launchers implemented in train_kernels.hip (storage: 0 fp32, 1 bf16) ----

// Hidden layer forward: Y = relu((A_hat X) W^k); with w_out != nullptr also
// t = Y w_out^k (the scalar layer's transform fused into the last hidden layer).
// partial_ready: the chunk partials of the pre-reduced rows for X are in heavy_partial
// already (bf16 storage only; otherwise a launch of its own computes them first).
void launch_fwd_hidden(const Launch& ln, int storage, int D, const GraphView& g, const void* X,
                       const float* W, int w_stride, void* Y, const float* w_out,
                       int wout_stride, float* t, float* heavy_partial, bool partial_ready = false);

// t = X w^k (used only when L = 1).
void launch_fwd_gemv(const Launch& ln, int storage, int D, const GraphView& g, const void* X,
                     const float* w, int w_stride, float* t);

// ---- width-1 kernels (narrow_kernels.hip) ----
// How the three passes run when each is a launch of its own and the gathered vector of a
// subgraph is first copied into LDS.  Workgroups of scalar_staged_waves() wavefronts;
// workgroup w works for subgraph wg_k[w] and is number w - wg_ptr[wg_k[w]] of the
// wg_ptr[k+1] - wg_ptr[k] that share subgraph k; cuts[w * waves + v] = range [x, y) of the
// light stream (whole rows) of its wavefront v; heavy_ptr[k .. k+1) = subgraph k's range in
// g.heavy_rows; cap = capacity of the LDS vector in floats, a multiple of 4, at least the
// largest subgraph's rows + 3 (the copy starts at a 16-byte boundary).  The grid has
// num_launch ids; id b stands for workgroup launch_of[b] (-1: none).  Loss partials: one per
// workgroup w.  Passing nullptr instead selects the form that gathers from memory
// (workgroups of decomposition WM_NARROW).
struct ScalarStaging {
  int num_launch = 0;
  int cap = 0;
  const int2* cuts = nullptr;
  const int* heavy_ptr = nullptr;
  const int* wg_k = nullptr;
  const int* wg_ptr = nullptr;
  const int* launch_of = nullptr;
};
int scalar_staged_waves();
int scalar_staged_max_cap();  // largest cap the kernel's one-round copy covers
size_t scalar_staged_lds_bytes(int cap);

// z = A_hat t, p = sigmoid(z).
void launch_fwd_readout(const Launch& ln, const GraphView& g, const float* t, float* z, float* p,
                        const ScalarStaging* sg);

// s = A_loc p; g_z = (c + q s) p (1 - p); loss partial per workgroup (g.num_loss_slots of them).
void launch_loss(const Launch& ln, const GraphView& g, const float* p, const float* c, float q,
                 float* g_z, double* loss_partial, const ScalarStaging* sg);

// For each of `sets` sets of workgroup partials (set s starts at loss_partial + s * set_stride):
// loss_part[s, k] = sum of the partials of subgraph k (if loss_part != nullptr);
// loss_out[s] = sum_k of those.  The training loop reduces many epochs with one launch.
void launch_loss_reduce(const Launch& ln, const GraphView& g, const double* loss_partial, int sets,
                        int64_t set_stride, double* loss_part, double* loss_out);
constexpr int kLossSets = 64;  // epochs whose loss partials are kept before they are reduced

// Best-by-loss snapshot (Alg. 1 stage 1).  `models` = number of weight sets: P (a subgraph
// with its own weights is a model) or 1 (shared weights: the batch is one model, judged by
// the total loss).  From one epoch's loss partials, summed as launch_loss_reduce sums
// them: improved[u] = 1 and best_loss[u], has_best[u] updated where model u was trained
// this epoch and its loss is below best_loss[u]; improved[u] = 0 otherwise.
void launch_best_update(const Launch& ln, const GraphView& g, const double* loss_partial, int models,
                        double* best_loss, int* improved, int* has_best);
// Copies the embedding rows (width D) and the weight tensors (w_elems[l] floats per model)
// of every model with flag[u] != 0 from *_src to *_dst.
void launch_param_copy(const Launch& ln, const GraphView& g, int models, int D, const int* flag,
                       const float* E_src, float* E_dst, const float* const* W_src, float* const* W_dst,
                       const int* w_elems, int num_w);

// The three width-1 passes in one launch, one workgroup of `waves` (4 or 16) wavefronts per
// subgraph; needs every subgraph's rows to fit the LDS (see scalar_fused_lds_bytes):
// p = sigmoid(A_hat t) [passes >= 1]; loss partial of subgraph k to loss_partial[k] and
// dL/dz kept in LDS [passes >= 2]; g_t = A_hat^T dL/dz [passes = 3].  cuts[k * waves + w] =
// range [x, y) of the light stream (whole rows) of wavefront w of subgraph k; heavy_ptr[k .. k+1) = subgraph k's range in
// g.heavy_rows; cap = row capacity of each of the two LDS vectors.  Subgraphs whose list in
// g.loss_ptr is empty are skipped.
size_t scalar_fused_lds_bytes(int waves, int cap);
void launch_scalar_fused(const Launch& ln, const GraphView& g, int waves, int cap, const int2* cuts,
                         const int* heavy_ptr, const float* t, float* p, const float* c, float q, float* g_t,
                         double* loss_partial, int passes);

// g_t = A_hat^T g_z.
void launch_bwd_readout(const Launch& ln, const GraphView& g, const float* g_z, float* g_t,
                        const ScalarStaging* sg);

// Backward of hidden layer l (and of the scalar layer when `last`):
//   last:  G_Z[j,:] = g_t[j] * w_out^k * [Hcur[j,:] > 0] is formed while gathering,
//          and gw_out partials = sum_i Hcur[i,:] g_t[i] are produced;
//   else:  G_Z is read from GZ_in.
//   G_T = A_hat^T G_Z;  gW partial += Hprev^T G_T;  G_Hprev = G_T W^T.
//   to_embed: Hprev is the embedding: apply `mode` (Adam / write gE / nothing);
//   else write GZ_out = G_Hprev * [Hprev > 0].
struct BwdArgs {
  const void* GZ_in = nullptr;   // [n, D] storage type (not last)
  void* GZ_last = nullptr;       // [n, D] bf16: where the wave-per-tile path forms G_Z of the last hidden layer
  const void* Hcur = nullptr;    // [n, D] storage type (last)
  const float* g_t = nullptr;    // [n] (last)
  const float* w_out = nullptr;  // [Pw, D] (last)
  int wout_stride = 0;
  float* gwout_partial = nullptr;  // [num_blocks, D] (last)
  const void* Hprev = nullptr;   // [n, D] storage type
  const float* W = nullptr;      // [Pw, D, D]
  int w_stride = 0;
  float* gW_partial = nullptr;   // [num_blocks, D*D]
  void* GZ_out = nullptr;        // [n, D] storage type (not to_embed)
  void* GT = nullptr;            // [n, D] bf16: rows of G_T = A_hat^T G_Z (wave-per-tile path, width 128)
  // to_embed
  int mode = EMBED_ADAM;
  float* E = nullptr;            // fp32 master embeddings [n, D]
  float* mE = nullptr;
  float* vE = nullptr;
  void* Eb = nullptr;            // bf16 working copy (bf16 storage only)
  float* gE = nullptr;           // EMBED_WRITE_GRAD
  AdamStep adam{};
  float* heavy_partial = nullptr;
};
void launch_bwd_hidden(const Launch& ln, int storage, int D, bool last, bool to_embed,
                       const GraphView& g, const BwdArgs& a);

// bf16-storage, matrix-core versions (layer_launch_bf16.hip, widths 64 and 128); `gt`
// already has the scale vectors of A_hat^T.
void launch_fwd_hidden_bf16(const Launch& ln, int D, const GraphView& g, const void* X, const float* W,
                            int w_stride, void* Y, const float* w_out, int wout_stride, float* t,
                            float* heavy_partial, bool partial_ready);
void launch_bwd_hidden_bf16(const Launch& ln, int D, bool last, bool to_embed, const GraphView& gt,
                            const BwdArgs& a);

// wave-per-tile bf16 kernels (wave_kernels_bf16.hip), widths 64 and 128
// last hidden layer: a.GZ_last = G_Z formed from g_t, w_out and Hcur; gw_out partials per
// narrow workgroup
void launch_form_gz_last(const Launch& ln, int D, const GraphView& g, const BwdArgs& a);
// hidden-layer backward on G_Z = a.GZ_in; gW partials per wave-kernel workgroup (width 64:
// of this kernel's own decomposition; width 128: of the hidden-backward decomposition,
// written by a second kernel from a.Hprev and the rows of G_T stored in a.GT)
void launch_bwd_hidden_wave(const Launch& ln, int D, bool to_embed, const GraphView& gt, const BwdArgs& a);
void launch_fwd_hidden_wave(const Launch& ln, int D, const GraphView& g, const void* X, const float* W,
                            int w_stride, void* Y, const float* w_out, int wout_stride, float* t,
                            float* heavy_partial);

// L = 1 backward: gw partial = sum_i X[i,:] g_t[i]; gE[i,:] = g_t[i] w^k.
void launch_bwd_single(const Launch& ln, int storage, int D, const GraphView& g, const BwdArgs& a);

// Sum the per-workgroup partials of each weight tensor in a fixed order, then
// apply Adam (or only write the gradient when grad_out != nullptr).  Up to three
// tensors (one per layer) are served by one launch.
struct WeightTensor {
  float* W = nullptr;
  float* m = nullptr;
  float* v = nullptr;
  const float* partial = nullptr;  // [workgroups, elems]
  const int* blk_ptr = nullptr;    // workgroups that hold partials of weight set kw:
  const int* blk_list = nullptr;   //   blk_list[blk_ptr[kw] .. blk_ptr[kw+1])
  float* grad_out = nullptr;       // [Pw, elems] or nullptr
  int elems = 0;                   // per subgraph
};
// many_partials: few weight sets with hundreds of partials each; the sum over a set's
// partials is then shared by 16 wavefronts per 64 weights.
// tail (bf16 storage, not with many_partials): the same launch also pre-reduces the chunks
// of the rows with very many neighbours of view g from the bf16 rows X into `partial`,
// ready for the next forward pass.
struct ChunkTail {
  GraphView g;
  const void* X = nullptr;
  float* partial = nullptr;
  int D = 0;
};
void launch_adam_w(const Launch& ln, int Pw, const WeightTensor* tensors, int count, const AdamStep& adam,
                   bool update, bool many_partials, const ChunkTail* tail = nullptr);  // adam.per_part, if set, is indexed by weight set; sets without partials are left alone

// fp32 -> bf16 copy (round to nearest even).
// X[i, :] <- softmax((X[i, :] - log(-log(U[i, :]))) / tau), rows of width D (Sec. 3.2).
void launch_gumbel_softmax_rows(const Launch& ln, int n, int D, float* X, const float* U, float tau);
void launch_to_bf16(const Launch& ln, const float* src, void* dst, int64_t count);
// bf16 -> fp32 copy (exact).
void launch_from_bf16(const Launch& ln, const void* src, float* dst, int64_t count);

// ---- launchers implemented in graph_kernels.hip ----

struct GraphBuildOut {
  int64_t nnz_local = 0;
  int64_t m_cut = 0;
  int error = 0;  // 0 ok; else a GCO_E* code with `message` set
  std::string message;
};

}  // namespace gco
