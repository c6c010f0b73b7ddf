// Host side of the C ABI declared in include/gco.h: argument checks, device
// memory, the static work decomposition, and the order of kernel launches that
// makes one training epoch (Sec. 3.2 of the paper) and the read-out steps
// (Sec. 3.3; Alg. 1 stages 2 and 3, first line).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <limits>
#include <string>
#include <queue>
#include <vector>

#include "gco.h"
#include "gco_internal.h"
#include "graph_kernels.h"

using namespace gco;

namespace {

const char* const kKindNames[KK_COUNT] = {
    "fwd_hidden", "fwd_gemv", "fwd_readout", "loss", "bwd_readout",
    "bwd_hidden", "bwd_embed_adam", "adam_w", "loss_reduce", "heavy_rows", "form_gz",
    "best_snapshot", "grad_w", "scalar_layer"};

struct EventPair {
  hipEvent_t a, b;
};

struct ProfilerImpl : Profiler {
  int mode = 0;
  uint64_t mask = ~0ull;
  std::vector<EventPair> pending[KK_COUNT];
  std::vector<EventPair> spare;
  int64_t launches[KK_COUNT] = {};
  double total_ms[KK_COUNT] = {};
  int64_t seen[KK_COUNT] = {};  // launches since the mode was set (mode 3 times one in kSampleEvery)
  bool open[KK_COUNT] = {};     // begin() recorded an event that end() has to close
  static constexpr int kSampleEvery = 8;
  bool on(int kind) const { return mode == 1 || (mode >= 2 && ((mask >> kind) & 1ull)); }
  void begin(int kind, hipStream_t st) override {
    if (!on(kind)) return;
    if (mode == 3 && (seen[kind]++ % kSampleEvery) != 0) return;
    EventPair ev;
    if (!spare.empty()) {
      ev = spare.back();
      spare.pop_back();
    } else {
      if (hipEventCreate(&ev.a) != hipSuccess || hipEventCreate(&ev.b) != hipSuccess) return;
    }
    (void)hipEventRecord(ev.a, st);
    pending[kind].push_back(ev);
    open[kind] = true;
  }
  void end(int kind, hipStream_t st) override {
    if (!open[kind]) return;
    (void)hipEventRecord(pending[kind].back().b, st);
    open[kind] = false;
  }
  void harvest() {  // the stream must be idle
    for (int k = 0; k < KK_COUNT; ++k) {
      for (EventPair& ev : pending[k]) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ev.a, ev.b) == hipSuccess) {
          total_ms[k] += ms;
          launches[k] += 1;
        }
        spare.push_back(ev);
      }
      pending[k].clear();
    }
  }
  void reset() {
    harvest();
    for (int k = 0; k < KK_COUNT; ++k) {
      launches[k] = 0;
      total_ms[k] = 0.0;
    }
  }
  ~ProfilerImpl() override {
    for (int k = 0; k < KK_COUNT; ++k)
      for (EventPair& ev : pending[k]) spare.push_back(ev);
    for (EventPair& ev : spare) {
      (void)hipEventDestroy(ev.a);
      (void)hipEventDestroy(ev.b);
    }
  }
};

}  // namespace

struct gco_ctx {
  gco_config cfg{};
  hipStream_t st = nullptr;
  std::string err;
  ProfilerImpl prof;

  // ---- graph ----
  bool has_graph = false;
  int n = 0, P = 1, Pw = 1;
  int64_t nnz_full = 0, nnz_loc = 0;
  int64_t* d_rowptr = nullptr;  // original order, full graph
  int32_t* d_col = nullptr;
  int32_t* d_part = nullptr;
  int32_t* d_perm = nullptr;    // new row -> original node
  int32_t* d_inv = nullptr;     // original node -> new row
  int32_t* d_lrowptr = nullptr; // local CSR, new order
  int32_t* d_lcol = nullptr;
  float *d_sa = nullptr, *d_sb = nullptr, *d_cbase = nullptr, *d_c = nullptr;
  int32_t* d_part_rows = nullptr;
  int32_t *d_blk_s = nullptr, *d_nblk_s = nullptr;
  int32_t *d_blk_S = nullptr, *d_nblk_S = nullptr;
  int32_t *d_heavy_of_row = nullptr, *d_heavy_chunk_ptr = nullptr, *d_chunk_begin = nullptr,
          *d_chunk_end = nullptr;
  int2* d_hpart = nullptr;
  int32_t *d_hpart_ptr = nullptr, *d_hpart_count = nullptr;
  float* d_hpart_partial = nullptr;
  int num_hparts = 0;
  int32_t* d_wrowptr = nullptr;
  // Everything that names which subgraph a unit of work belongs to, on the host (as built
  // at upload) and on the device twice: for all subgraphs (`full`) and for the subset of
  // the current gco_train_subset call (`sub`, units of the other subgraphs marked -1).
  struct HostMaps {
    std::vector<int> blk_k, nblk_k, wblk_k[kWaveMaps], chunk_part, heavy_rows, heavy_part, staged_k;
  } hm;
  struct ActiveMaps {
    int32_t *blk_k = nullptr, *nblk_k = nullptr, *wblk_k[kWaveMaps] = {}, *chunk_part = nullptr,
            *heavy_rows = nullptr;
    // workgroups that hold partials, per weight set: wide kernels, wave kernels, narrow tiles
    int32_t *pbl_ptr = nullptr, *pbl_list = nullptr;
    int32_t *wpbl_ptr[kWaveMaps] = {}, *wpbl_list[kWaveMaps] = {};
    int32_t *nwbl_ptr = nullptr, *nwbl_list = nullptr;
    // loss partial slots per subgraph
    int32_t *loss_ptr = nullptr, *loss_list = nullptr;
    bool allocated = false;
  } full, sub;
  GraphView gv_sub;
  std::vector<uint8_t> sub_active;  // the subset `sub` was built for
  int num_wblocks[kWaveMaps] = {};
  int num_loss_slots = 0;
  // the three width-1 passes as one launch with a workgroup per subgraph: possible when
  // two float vectors of the largest subgraph fit the LDS of a compute unit
  bool fused_scalar = false;
  int fused_waves = 0, fused_cap = 0;
  // the three width-1 passes as three launches that copy the gathered vector into LDS first
  bool staged_scalar = false;
  int staged_wgs = 0, staged_cap = 0;
  int32_t *d_staged_k = nullptr, *d_staged_ptr = nullptr, *d_staged_launch = nullptr;
  int scalar_form_wanted = GCO_SCALAR_AUTO;
  int2* d_fused_cuts = nullptr;
  int32_t* d_heavy_ptr = nullptr;
  WaveRun* d_wave_runs[kWaveMaps] = {};
  int2 *d_went = nullptr, *d_went_t = nullptr;
  float *d_wval = nullptr, *d_wval_t = nullptr;
  int32_t* d_wrowid = nullptr;
  int32_t* d_wtile_hptr = nullptr;
  int2 *d_ent = nullptr, *d_ent_t = nullptr;
  float* d_diag = nullptr;
  float* d_heavy_partial = nullptr;
  // chunk partials of the pre-reduced rows for the FIRST layer (from the bf16 working copy of
  // the embeddings), written by the last launch of an epoch for the next one; valid while
  // they belong to the current embeddings of every subgraph
  float* d_heavy_partial_E = nullptr;
  bool heavy_E_valid = false;
  GraphView gv;
  std::vector<void*> graph_allocs;

  // ---- parameters and activations (new order) ----
  bool has_params = false;
  bool probs_valid = false;
  // Adam step counts: one per subgraph (embedding rows) and one per weight set
  std::vector<int64_t> stepE, stepW;
  float2* d_bc = nullptr;  // bias corrections of up to kLossSets epochs, [epoch][P + Pw]
  float *E = nullptr, *mE = nullptr, *vE = nullptr;
  void* Eb = nullptr;
  float *W[3] = {}, *mW[3] = {}, *vW[3] = {};
  float* gW_partial[3] = {};  // [l-1] for hidden layers; the scalar layer uses gwout_partial
  float* gwout_partial = nullptr;
  void* H[3] = {};            // H[0] aliases the embedding in storage type
  void* GZ[3] = {};
  void* GT = nullptr;         // rows of A_hat^T G_Z of the layer in hand (split_grad_w())
  float *t = nullptr, *z = nullptr, *p = nullptr, *g_z = nullptr, *g_t = nullptr;
  double *loss_partial = nullptr, *loss_part = nullptr, *loss_hist = nullptr, *loss_one = nullptr;
  int64_t loss_hist_cap = 0;

  // best-by-loss snapshot: one model per weight set (Pw of them)
  bool best_on = false, best_alloc = false;
  float* E_best = nullptr;
  float* W_best[3] = {};
  double* d_best_loss = nullptr;
  int32_t *d_improved = nullptr, *d_has_best = nullptr;

  double kind_bytes[KK_COUNT] = {};

  int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    err = buf;
    return code;
  }

  void* raw_alloc(size_t bytes) {
    if (bytes == 0) bytes = 256;
    if (cfg.dev_alloc) return cfg.dev_alloc(bytes, cfg.alloc_user);
    void* ptr = nullptr;
    if (hipMalloc(&ptr, bytes) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    return ptr;
  }
  void raw_free(void* ptr) {
    if (!ptr) return;
    if (cfg.dev_free) cfg.dev_free(ptr, cfg.alloc_user);
    else (void)hipFree(ptr);
  }
  template <typename T>
  bool galloc(T** out, size_t count) {
    void* ptr = raw_alloc(count * sizeof(T));
    if (!ptr) return false;
    graph_allocs.push_back(ptr);
    *out = static_cast<T*>(ptr);
    return true;
  }
  void free_graph() {
    (void)hipStreamSynchronize(st);
    prof.harvest();
    for (void* q : graph_allocs) raw_free(q);
    graph_allocs.clear();
    has_graph = has_params = probs_valid = false;
    heavy_E_valid = false;
    num_hparts = 0;
    best_on = best_alloc = false;
    loss_hist_cap = 0;
    loss_hist = nullptr;
  }
  int elem_bytes() const { return cfg.storage == GCO_STORAGE_BF16 ? 2 : 4; }
  // the hidden layers run on the wave-per-tile kernels (bf16 storage: width 64 or 128)
  bool wave_path() const { return cfg.storage == GCO_STORAGE_BF16; }
  // width 128: the weight gradients come from a kernel of their own, fed with stored G_T rows
  bool split_grad_w() const { return wave_path() && cfg.dim == 128; }
  // decomposition whose workgroups wrote the weight-gradient partials of hidden layer l
  int grad_map(int l) const { return split_grad_w() ? WM_GRADW : (l == 1 ? WM_EMBED : WM_BWD); }
  Launch launch() { return Launch{st, prof.mode ? &prof : nullptr}; }
};

#define HIPCHK(expr)                                                                   \
  do {                                                                                 \
    hipError_t e_ = (expr);                                                            \
    if (e_ != hipSuccess)                                                              \
      return ctx->fail(GCO_EDEVICE, "%s failed: %s", #expr, hipGetErrorString(e_));    \
  } while (0)

#define NEED(cond, code, ...) \
  do {                        \
    if (!(cond)) return ctx->fail(code, __VA_ARGS__); \
  } while (0)

#define GALLOC(ptr, count)                                                              \
  do {                                                                                  \
    if (!ctx->galloc(&(ptr), (count)))                                                  \
      return ctx->fail(GCO_ENOMEM, "device allocation of %zu bytes failed (%s)",        \
                       static_cast<size_t>(count) * sizeof(*(ptr)), #ptr);              \
  } while (0)

namespace {

// RAII for short-lived device scratch of one call.
struct Scratch {
  gco_ctx* ctx;
  std::vector<void*> ptrs;
  explicit Scratch(gco_ctx* c) : ctx(c) {}
  template <typename T>
  T* get(size_t count) {
    void* q = ctx->raw_alloc(count * sizeof(T));
    if (q) ptrs.push_back(q);
    return static_cast<T*>(q);
  }
  ~Scratch() {
    (void)hipStreamSynchronize(ctx->st);
    for (void* q : ptrs) ctx->raw_free(q);
  }
};

template <typename T>
hipError_t h2d(gco_ctx* ctx, T* dst, const T* src, size_t count) {
  if (count == 0) return hipSuccess;
  hipError_t e = hipMemcpyAsync(dst, src, count * sizeof(T), hipMemcpyHostToDevice, ctx->st);
  if (e != hipSuccess) return e;
  return hipStreamSynchronize(ctx->st);  // the host buffer belongs to the caller again on return
}
template <typename T>
hipError_t d2h(gco_ctx* ctx, T* dst, const T* src, size_t count) {
  if (count == 0) return hipStreamSynchronize(ctx->st);
  hipError_t e = hipMemcpyAsync(dst, src, count * sizeof(T), hipMemcpyDeviceToHost, ctx->st);
  if (e != hipSuccess) return e;
  return hipStreamSynchronize(ctx->st);
}

int w_elems(const gco_ctx* ctx, int l /*1..L*/) {
  const int D = ctx->cfg.dim;
  return l < ctx->cfg.num_layers ? D * D : D;
}

// Workgroup -> (subgraph k, first tile s, stride S_k) tables: workgroup b walks
// tiles s, s + S_k, s + 2 S_k, ... of subgraph k.  S_k is proportional to the
// subgraph's share of the work (rows and CSR entries), at least
// ceil(tiles_k / max_tiles_per_block), at most tiles_k.  With group_by_xcd, all
// workgroups of a subgraph get ids that are equal modulo 8, so that they land on
// one XCD and share its L2 (workgroups are dealt to the 8 XCDs round-robin by id);
// subgraphs are spread over the XCDs longest-first.  The caller asks for that when
// the feature matrix does not fit the Infinity Cache: while it fits, grouping gains
// nothing measurable (c4: 0.977 against 0.973 ms per epoch) and costs the balance of
// runs in which only some subgraphs train.
// Shares of `target` units in proportion to work[k], share k within [lo[k], hi[k]].  The
// shares add up to exactly `target` whenever the bounds allow it: a launch sized to a whole
// number of rounds of resident workgroups must not spill a handful of workgroups into one
// more round (measured at c4: 1538 instead of 1532 forward workgroups, 768 resident, cost
// 6 % of the launch).  Units are added where the work per unit is largest and taken away
// where it is smallest; ties go to the lower index.
std::vector<int> apportion(const std::vector<double>& work, int64_t target, const std::vector<int>& lo,
                           const std::vector<int>& hi) {
  const int P = static_cast<int>(work.size());
  double total = 0;
  for (double w : work) total += w;
  std::vector<int> share(P);
  int64_t sum = 0;
  for (int k = 0; k < P; ++k) {
    const double want = total > 0 ? std::floor(static_cast<double>(target) * work[k] / total) : 0.0;
    share[k] = std::max(lo[k], std::min(hi[k], static_cast<int>(want)));
    sum += share[k];
  }
  using Item = std::pair<double, int>;  // (work per unit, -k): the heap's top is the largest
  if (sum < target) {
    std::priority_queue<Item> q;
    for (int k = 0; k < P; ++k)
      if (share[k] < hi[k]) q.push({work[k] / (share[k] + 1), -k});
    while (sum < target && !q.empty()) {
      const int k = -q.top().second;
      q.pop();
      ++share[k];
      ++sum;
      if (share[k] < hi[k]) q.push({work[k] / (share[k] + 1), -k});
    }
  } else if (sum > target) {
    std::priority_queue<Item> q;  // smallest work per unit first: keys negated
    for (int k = 0; k < P; ++k)
      if (share[k] > lo[k]) q.push({-work[k] / share[k], -k});
    while (sum > target && !q.empty()) {
      const int k = -q.top().second;
      q.pop();
      --share[k];
      --sum;
      if (share[k] > lo[k]) q.push({-work[k] / share[k], -k});
    }
  }
  return share;
}

void build_block_map(int P, const std::vector<int>& part_rows, const std::vector<int32_t>& lrowptr,
                     int tile_rows, int target_blocks, int max_tiles_per_block,
                     std::vector<int>& blk_k, std::vector<int>& blk_s, std::vector<int>& blk_S,
                     bool group_by_xcd, double row_cost = 2.0, const std::vector<double>* entries_of = nullptr) {
  // entries_of: the entries a subgraph's workgroups walk, where that is not every local
  // neighbour (the wave kernels leave the rows with very many neighbours to other workgroups)
  std::vector<int> tiles(P), Sk(P);
  std::vector<double> work(P);
  for (int k = 0; k < P; ++k) {
    const int rows = part_rows[k + 1] - part_rows[k];
    tiles[k] = (rows + tile_rows - 1) / tile_rows;
    work[k] = row_cost * rows +
              (entries_of ? (*entries_of)[k] : static_cast<double>(lrowptr[part_rows[k + 1]] - lrowptr[part_rows[k]]));
  }
  {
    std::vector<int> lo(P), hi(P);
    for (int k = 0; k < P; ++k) {
      lo[k] = tiles[k] == 0 ? 0 : 1;
      if (max_tiles_per_block > 0) lo[k] = std::max(lo[k], (tiles[k] + max_tiles_per_block - 1) / max_tiles_per_block);
      hi[k] = std::max(lo[k], tiles[k]);
    }
    Sk = apportion(work, target_blocks, lo, hi);
  }
  blk_k.clear();
  blk_s.clear();
  blk_S.clear();
  if (group_by_xcd && P >= 8) {
    std::vector<int> order(P);
    for (int k = 0; k < P; ++k) order[k] = k;
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return Sk[x] > Sk[y]; });
    std::vector<std::vector<int>> per_xcd(8);   // unit = k * 2^? not needed: store (k, s) pairs flat
    std::vector<std::vector<int>> per_xcd_s(8);
    for (int k : order) {
      int best = 0;
      for (int x = 1; x < 8; ++x)
        if (per_xcd[x].size() < per_xcd[best].size()) best = x;
      for (int sidx = 0; sidx < Sk[k]; ++sidx) {
        per_xcd[best].push_back(k);
        per_xcd_s[best].push_back(sidx);
      }
    }
    size_t depth = 0;
    for (int x = 0; x < 8; ++x) depth = std::max(depth, per_xcd[x].size());
    blk_k.assign(depth * 8, -1);
    blk_s.assign(depth * 8, 0);
    blk_S.assign(depth * 8, 1);
    for (int x = 0; x < 8; ++x)
      for (size_t q = 0; q < per_xcd[x].size(); ++q) {
        const size_t b = q * 8 + x;
        blk_k[b] = per_xcd[x][q];
        blk_s[b] = per_xcd_s[x][q];
        blk_S[b] = Sk[per_xcd[x][q]];
      }
  } else {
    for (int k = 0; k < P; ++k)
      for (int sidx = 0; sidx < Sk[k]; ++sidx) {
        blk_k.push_back(k);
        blk_s.push_back(sidx);
        blk_S.push_back(Sk[k]);
      }
  }
  if (blk_k.empty()) {  // keep the grid non-empty
    blk_k.push_back(-1);
    blk_s.push_back(0);
    blk_S.push_back(1);
  }
}

// Wave-per-tile kernels: workgroups are dealt to the subgraphs as above; the tiles of a
// subgraph (kWaveRows rows each) are then cut into one contiguous run per wavefront such
// that every run costs about the same: a tile costs its light-stream entries (one per row
// plus the neighbours of rows that are not pre-reduced) plus row_cost per row, which
// stands for the per-row work of the kernel's dense part and epilogue.
void build_wave_map(int P, const std::vector<int>& part_rows, const std::vector<int32_t>& lrowptr,
                    int target_blocks, double row_cost, bool group_by_xcd, std::vector<int>& wblk_k,
                    std::vector<WaveRun>& wave_runs) {
  constexpr int kWaves = kBlock / 64;
  std::vector<int> blk_s, blk_S;
  // the subgraphs' shares follow the same cost as the cuts below: the light stream's entries
  // (the neighbours of pre-reduced rows are summed elsewhere) plus row_cost per row
  std::vector<double> light(static_cast<size_t>(P), 0.0);
  for (int k = 0; k < P; ++k)
    for (int r = part_rows[k]; r < part_rows[k + 1]; ++r) {
      const int deg = lrowptr[r + 1] - lrowptr[r];
      light[k] += 1 + (deg >= kHeavyMin ? 0 : deg);
    }
  build_block_map(P, part_rows, lrowptr, kWaveRows * kWaves, target_blocks, 0, wblk_k, blk_s, blk_S,
                  group_by_xcd, row_cost, &light);
  wave_runs.assign(wblk_k.size() * kWaves, WaveRun{});
  // light-stream offset of every row (one entry per row plus the neighbours of rows that
  // are not pre-reduced) and global number of every subgraph's first tile
  const int n = part_rows[P];
  std::vector<int> wrow(static_cast<size_t>(n) + 1, 0), tbase(static_cast<size_t>(P) + 1, 0);
  for (int r = 0; r < n; ++r) {
    const int deg = lrowptr[r + 1] - lrowptr[r];
    wrow[r + 1] = wrow[r] + 1 + (deg >= kHeavyMin ? 0 : deg);
  }
  for (int k = 0; k < P; ++k)
    tbase[k + 1] = tbase[k] + (part_rows[k + 1] - part_rows[k] + kWaveRows - 1) / kWaveRows;
  std::vector<std::vector<int>> cuts(P);  // cuts[k][v] = first tile of wavefront v of subgraph k
  for (size_t b = 0; b < wblk_k.size(); ++b) {
    const int k = wblk_k[b];
    if (k < 0) continue;
    if (cuts[k].empty()) {
      const int rows = part_rows[k + 1] - part_rows[k];
      const int tiles = (rows + kWaveRows - 1) / kWaveRows;
      std::vector<double> pre(static_cast<size_t>(tiles) + 1, 0);  // cost before tile t
      for (int t = 0; t < tiles; ++t) {
        double c = row_cost * kWaveRows;
        for (int r = part_rows[k] + t * kWaveRows; r < std::min(part_rows[k + 1], part_rows[k] + (t + 1) * kWaveRows); ++r) {
          const int deg = lrowptr[r + 1] - lrowptr[r];
          c += 1 + (deg >= kHeavyMin ? 0 : deg);
        }
        pre[t + 1] = pre[t] + c;
      }
      const int V = blk_S[b] * kWaves;
      cuts[k].assign(static_cast<size_t>(V) + 1, tiles);
      cuts[k][0] = 0;
      int t = 0;
      for (int v = 1; v < V; ++v) {
        const double want = pre[tiles] * v / V;
        while (t < tiles && pre[t] < want) ++t;
        cuts[k][v] = t;
      }
    }
    for (int q = 0; q < kWaves; ++q) {
      const int v = blk_s[b] * kWaves + q;
      WaveRun& run = wave_runs[b * kWaves + q];
      run.tile0 = cuts[k][v];
      run.tile1 = cuts[k][v + 1];
      run.rbeg = part_rows[k];
      run.rend = part_rows[k + 1];
      run.e0 = wrow[std::min(run.rend, run.rbeg + run.tile0 * kWaveRows)];
      run.e1 = wrow[std::min(run.rend, run.rbeg + run.tile1 * kWaveRows)];
      run.tglob = tbase[k];
    }
  }
}

// Workgroup ids grouped by the subgraph they work on (ascending within a group);
// with num_sets == 1 every valid workgroup goes to the single group.
void bucket_blocks(const std::vector<int>& blk_k, int num_sets, std::vector<int>& ptr,
                   std::vector<int>& list) {
  ptr.assign(num_sets + 1, 0);
  for (int k : blk_k)
    if (k >= 0) ptr[(num_sets == 1 ? 0 : k) + 1]++;
  for (int q = 0; q < num_sets; ++q) ptr[q + 1] += ptr[q];
  list.assign(static_cast<size_t>(ptr[num_sets]), 0);
  std::vector<int> cursor(ptr.begin(), ptr.end() - 1);
  for (size_t b = 0; b < blk_k.size(); ++b)
    if (blk_k[b] >= 0) list[cursor[num_sets == 1 ? 0 : blk_k[b]]++] = static_cast<int>(b);
}

// Builds the subgraph-naming arrays of `m` from the host copies: units of subgraphs with
// active[k] == 0 are marked -1 and left out of the lists (active == nullptr: all take part).
int upload_active_maps(gco_ctx* ctx, gco_ctx::ActiveMaps& m, const uint8_t* active) {
  const gco_ctx::HostMaps& h = ctx->hm;
  const int P = ctx->P, Pw = ctx->Pw;
  auto filtered = [&](const std::vector<int>& src) {
    std::vector<int> out(src);
    if (active != nullptr)
      for (int& k : out)
        if (k >= 0 && !active[k]) k = -1;
    return out;
  };
  const bool first = !m.allocated;
  auto put = [&](int32_t*& dst, const std::vector<int>& v, size_t capacity) -> int {
    if (first) GALLOC(dst, std::max<size_t>(1, capacity));
    HIPCHK(h2d(ctx, dst, v.data(), v.size()));
    return GCO_OK;
  };
  auto put_lists = [&](int32_t*& ptr, int32_t*& list, const std::vector<int>& ks, int sets) -> int {
    std::vector<int> pv, lv;
    bucket_blocks(ks, sets, pv, lv);
    int rc = put(ptr, pv, pv.size());
    if (rc != GCO_OK) return rc;
    return put(list, lv, ks.size());
  };
#define PUT(expr)                 \
  do {                            \
    const int rc_ = (expr);       \
    if (rc_ != GCO_OK) return rc_; \
  } while (0)
  const std::vector<int> blk_k = filtered(h.blk_k), nblk_k = filtered(h.nblk_k);
  PUT(put(m.blk_k, blk_k, blk_k.size()));
  PUT(put(m.nblk_k, nblk_k, nblk_k.size()));
  PUT(put_lists(m.pbl_ptr, m.pbl_list, blk_k, Pw));
  PUT(put_lists(m.nwbl_ptr, m.nwbl_list, nblk_k, Pw));
  std::vector<int> narrow;
  for (int v = 0; v < kWaveMaps; ++v) {
    const std::vector<int> wk = filtered(h.wblk_k[v]);
    PUT(put(m.wblk_k[v], wk, wk.size()));
    PUT(put_lists(m.wpbl_ptr[v], m.wpbl_list[v], wk, Pw));
    if (v == WM_NARROW) narrow = wk;
  }
  const std::vector<int> chunk_part = filtered(h.chunk_part), heavy_part = filtered(h.heavy_part);
  PUT(put(m.chunk_part, chunk_part, chunk_part.size()));
  std::vector<int> heavy_rows(h.heavy_rows);
  for (size_t q = 0; q < heavy_rows.size(); ++q)
    if (heavy_part[q] < 0) heavy_rows[q] = -1;
  PUT(put(m.heavy_rows, heavy_rows, heavy_rows.size()));
  // loss partial slots: one per pre-reduced row, then one per workgroup of the width-1
  // kernels; with the one-launch scalar layer, one per subgraph; with the staged form, one
  // per workgroup of those launches
  std::vector<int> slot_k(heavy_part);
  slot_k.insert(slot_k.end(), narrow.begin(), narrow.end());
  if (ctx->fused_scalar || ctx->staged_scalar) {
    slot_k = h.staged_k;  // subgraph of every workgroup of that launch
    for (int& k : slot_k)
      if (active != nullptr && !active[k]) k = -1;
  }
  PUT(put_lists(m.loss_ptr, m.loss_list, slot_k, P));
#undef PUT
  m.allocated = true;
  return GCO_OK;
}

// The graph view with the subgraph-naming arrays of `m`.
GraphView view_with(const gco_ctx* ctx, const gco_ctx::ActiveMaps& m) {
  GraphView g = ctx->gv;
  g.blk_k = m.blk_k;
  g.nblk_k = m.nblk_k;
  for (int v = 0; v < kWaveMaps; ++v) g.wblk_k[v] = m.wblk_k[v];
  g.chunk_part = m.chunk_part;
  g.heavy_rows = m.heavy_rows;
  g.loss_ptr = m.loss_ptr;
  g.loss_list = m.loss_list;
  return g;
}

// Algorithmic bytes per launch of every kernel kind: each array of the METHOD that the
// kernel reads or writes, once (gathers taken as cache-served).  Buffers that exist only
// because of how the work is cut up (per-workgroup partial sums of the weight gradients and
// of the loss, chunk partials of pre-reduced rows) are not counted.
void traffic_model(gco_ctx* ctx) {
  const double n = ctx->n, nnz = static_cast<double>(ctx->nnz_loc), D = ctx->cfg.dim;
  const double s = ctx->elem_bytes(), Pw = ctx->Pw;
  const int L = ctx->cfg.num_layers;
  const double idx = nnz * 4 + (n + 1) * 4, scales = 2 * n * 4;
  double* kb = ctx->kind_bytes;
  for (int k = 0; k < KK_COUNT; ++k) kb[k] = 0;
  // hidden forward: X read + Y write + W (+ t and w_out on the last hidden layer; averaged)
  if (L >= 2) {
    const double base = idx + scales + 2 * n * D * s + Pw * D * D * 4;
    kb[KK_FWD_HIDDEN] = base + (n * 4 + Pw * D * 4) / (L - 1);
  }
  kb[KK_FWD_GEMV] = n * D * s + Pw * D * 4 + n * 4;
  kb[KK_FWD_READOUT] = idx + scales + 3 * n * 4;
  kb[KK_LOSS] = idx + 3 * n * 4;
  kb[KK_BWD_READOUT] = idx + scales + 2 * n * 4;
  // the three passes in one launch: t and c in, p and g_t out; z and dL/dz never travel
  kb[KK_SCALAR_FUSED] = 3 * idx + 2 * scales + 4 * n * 4;
  // On the wave-per-tile path G_Z of the last hidden layer is formed by a kernel of its own
  // (KK_FORM_GZ) instead of inside the layer's backward.
  const bool wave = ctx->wave_path() && L >= 2;
  const bool split = ctx->split_grad_w() && L >= 2;
  const double last_extra = wave ? 0 : n * 4;  // g_t read
  if (wave) kb[KK_FORM_GZ] = 2 * n * D * s + n * 4 + Pw * D * 4;
  // gathered gradient source + Hprev read + GZ write + W (the weight gradient itself: Pw D^2)
  kb[KK_BWD_HIDDEN] = idx + scales + 3 * n * D * s + 2 * Pw * D * D * 4 + (L == 3 ? last_extra : 0);
  if (split) {
    // the weight gradient moves to grad_w, which reads Hprev and the stored rows of G_T
    kb[KK_BWD_HIDDEN] += n * D * s - Pw * D * D * 4;
    kb[KK_GRAD_W] = 2 * n * D * s + Pw * D * D * 4;
  }
  // first layer: gathered source + embedding (working copy) read + Adam state in/out
  const double adam_e = ctx->cfg.train_embed ? (6 * n * D * 4 + (s == 2 ? n * D * 2 : 0)) : 0;
  const double hprev_read = (s == 2 || !ctx->cfg.train_embed) ? n * D * s : 0;  // fp32: E is read by Adam already
  if (L >= 2 && split)  // gathered source + G_T rows out + Adam; the working copy is read by grad_w
    kb[KK_BWD_EMBED] = idx + scales + 2 * n * D * s + Pw * D * D * 4 + adam_e;
  else if (L >= 2)
    kb[KK_BWD_EMBED] = idx + scales + n * D * s + hprev_read + 2 * Pw * D * D * 4 + adam_e +
                       (L == 2 ? last_extra : 0);
  else
    kb[KK_BWD_EMBED] = n * 4 + hprev_read + adam_e + Pw * D * 4;
  // one launch serves all weight tensors: the gradient in, W, m, v in and out
  double wtot = 0;
  for (int l = 1; l <= L; ++l) {
    const double e = l < L ? D * D : D;
    wtot += Pw * e * 28;
  }
  kb[KK_ADAM_W] = wtot;
  kb[KK_LOSS_REDUCE] = ctx->P * 8.0;
  kb[KK_HEAVY] = 0;  // reported by time only
  kb[KK_BEST] = 0;   // depends on how many models improved
  if (!split) kb[KK_GRAD_W] = 0;
}

}  // namespace

// =============================================================================
// C ABI
// =============================================================================
extern "C" {

int gco_default_config(gco_config* cfg) {
  if (!cfg) return GCO_EINVAL;
  std::memset(cfg, 0, sizeof *cfg);
  cfg->problem = GCO_PROBLEM_MIS;
  cfg->num_layers = 2;
  cfg->dim = 16;
  cfg->norm = GCO_NORM_SYM;
  cfg->storage = GCO_STORAGE_FP32;
  cfg->weight_sharing = 0;
  cfg->train_embed = 1;
  cfg->alpha = 2.f;
  cfg->beta = 1.f;
  cfg->lr = 1e-2f;
  cfg->adam_b1 = 0.9f;
  cfg->adam_b2 = 0.999f;
  cfg->adam_eps = 1e-8f;
  return GCO_OK;
}

int gco_create(const gco_config* cfg, gco_ctx** out) {
  if (!cfg || !out) return GCO_EINVAL;
  *out = nullptr;
  const int D = cfg->dim;
  const bool dim_ok = D == 8 || D == 16 || D == 32 || D == 64 || D == 128;
  if (!dim_ok || cfg->num_layers < 1 || cfg->num_layers > 3) return GCO_EINVAL;
  if (cfg->problem != GCO_PROBLEM_MIS && cfg->problem != GCO_PROBLEM_MAXCUT) return GCO_EINVAL;
  if (cfg->norm != GCO_NORM_SYM && cfg->norm != GCO_NORM_MEAN) return GCO_EINVAL;
  if (cfg->storage != GCO_STORAGE_FP32 && cfg->storage != GCO_STORAGE_BF16) return GCO_EINVAL;
  if (cfg->storage == GCO_STORAGE_BF16 && D != 64 && D != 128) return GCO_EINVAL;
  if ((cfg->dev_alloc == nullptr) != (cfg->dev_free == nullptr)) return GCO_EINVAL;
  if (!(cfg->lr > 0.f) || !(cfg->adam_b1 >= 0.f && cfg->adam_b1 < 1.f) ||
      !(cfg->adam_b2 >= 0.f && cfg->adam_b2 < 1.f) || !(cfg->adam_eps > 0.f))
    return GCO_EINVAL;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return GCO_EDEVICE;
  }
  gco_ctx* ctx = new (std::nothrow) gco_ctx();
  if (!ctx) return GCO_ENOMEM;
  ctx->cfg = *cfg;
  ctx->st = static_cast<hipStream_t>(cfg->stream);
  *out = ctx;
  return GCO_OK;
}

int gco_destroy(gco_ctx* ctx) {
  if (!ctx) return GCO_EINVAL;
  ctx->free_graph();
  delete ctx;
  return GCO_OK;
}

int gco_get_config(gco_ctx* ctx, gco_config* out) {
  if (!ctx || !out) return GCO_EINVAL;
  *out = ctx->cfg;
  return GCO_OK;
}

int gco_set_scalar_layer_form(gco_ctx* ctx, int form) {
  if (!ctx) return GCO_EINVAL;
  NEED(form >= GCO_SCALAR_AUTO && form <= GCO_SCALAR_ONE_LAUNCH, GCO_EINVAL, "unknown scalar-layer form %d", form);
  ctx->scalar_form_wanted = form;
  return GCO_OK;
}

int gco_get_scalar_layer_form(gco_ctx* ctx, int* form) {
  if (!ctx || !form) return GCO_EINVAL;
  NEED(ctx->has_graph, GCO_ESTATE, "no graph uploaded");
  *form = ctx->fused_scalar ? GCO_SCALAR_ONE_LAUNCH : ctx->staged_scalar ? GCO_SCALAR_STAGED : GCO_SCALAR_STREAMS;
  return GCO_OK;
}

const char* gco_last_error(gco_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int gco_sync(gco_ctx* ctx) {
  if (!ctx) return GCO_EINVAL;
  HIPCHK(hipStreamSynchronize(ctx->st));
  return GCO_OK;
}

int gco_upload_graph(gco_ctx* ctx, int64_t n64, const int64_t* rowptr, const int32_t* col,
                     const int32_t* part_id, int32_t num_parts) {
  if (!ctx) return GCO_EINVAL;
  NEED(rowptr != nullptr, GCO_EINVAL, "rowptr is NULL");
  NEED(n64 >= 1 && n64 < std::numeric_limits<int32_t>::max(), GCO_ERANGE, "n = %lld out of range",
       static_cast<long long>(n64));
  const int n = static_cast<int>(n64);
  if (!part_id) num_parts = 1;
  NEED(num_parts >= 1 && num_parts <= n, GCO_EINVAL, "num_parts = %d not in [1, n]", num_parts);
  // the per-subgraph loss sums of an epoch are held in one workgroup's LDS
  NEED(num_parts <= kMaxParts, GCO_ERANGE, "num_parts = %d exceeds %d (merge small subgraphs, e.g. gco_pack_parts)",
       num_parts, kMaxParts);
  NEED(rowptr[0] == 0, GCO_EINVAL, "rowptr[0] != 0");
  for (int i = 0; i < n; ++i)
    NEED(rowptr[i + 1] >= rowptr[i], GCO_EINVAL, "rowptr decreases at row %d", i);
  const int64_t nnz = rowptr[n];
  NEED(nnz == 0 || col != nullptr, GCO_EINVAL, "col is NULL");
  NEED(nnz % 2 == 0, GCO_EINVAL, "odd number of CSR entries: not a symmetric graph");
  const int P = num_parts;
  std::vector<int> part_rows(P + 1, 0);
  if (part_id) {
    for (int i = 0; i < n; ++i) {
      NEED(part_id[i] >= 0 && part_id[i] < P, GCO_EINVAL, "part_id[%d] = %d not in [0, %d)", i,
           part_id[i], P);
      part_rows[part_id[i] + 1]++;
    }
  } else {
    part_rows[1] = n;
  }
  for (int k = 0; k < P; ++k) part_rows[k + 1] += part_rows[k];

  ctx->free_graph();
  ctx->n = n;
  ctx->P = P;
  ctx->Pw = ctx->cfg.weight_sharing ? 1 : P;
  ctx->nnz_full = nnz;
  const int D = ctx->cfg.dim;
  const int L = ctx->cfg.num_layers;
  hipStream_t st = ctx->st;

  // stable counting sort by subgraph id: perm (new -> original), inv (original -> new)
  std::vector<int32_t> perm(n), inv(n);
  {
    std::vector<int> cursor(part_rows.begin(), part_rows.end() - 1);
    for (int i = 0; i < n; ++i) {
      const int k = part_id ? part_id[i] : 0;
      const int r = cursor[k]++;
      perm[r] = i;
      inv[i] = r;
    }
  }

  GALLOC(ctx->d_rowptr, static_cast<size_t>(n) + 1);
  GALLOC(ctx->d_col, static_cast<size_t>(nnz));
  GALLOC(ctx->d_part, static_cast<size_t>(n));
  GALLOC(ctx->d_perm, static_cast<size_t>(n));
  GALLOC(ctx->d_inv, static_cast<size_t>(n));
  GALLOC(ctx->d_part_rows, static_cast<size_t>(P) + 1);
  HIPCHK(h2d(ctx, ctx->d_rowptr, rowptr, static_cast<size_t>(n) + 1));
  HIPCHK(h2d(ctx, ctx->d_col, col, static_cast<size_t>(nnz)));
  if (part_id) {
    HIPCHK(h2d(ctx, ctx->d_part, part_id, static_cast<size_t>(n)));
  } else {
    launch_fill_u32(st, ctx->d_part, n, 0u);
  }
  HIPCHK(h2d(ctx, ctx->d_perm, perm.data(), perm.size()));
  HIPCHK(h2d(ctx, ctx->d_inv, inv.data(), inv.size()));
  HIPCHK(h2d(ctx, ctx->d_part_rows, part_rows.data(), part_rows.size()));

  std::vector<int32_t> lrowptr(static_cast<size_t>(n) + 1);
  {
    Scratch tmp(ctx);
    int* d_err = tmp.get<int>(1);
    int64_t* d_count = tmp.get<int64_t>(static_cast<size_t>(n) + 1);
    int64_t* d_lptr64 = tmp.get<int64_t>(static_cast<size_t>(n) + 1);
    int64_t* d_scan = tmp.get<int64_t>(scan_temp_elems(static_cast<int64_t>(n) + 1));
    NEED(d_err && d_count && d_lptr64 && d_scan, GCO_ENOMEM, "device scratch allocation failed");
    launch_fill_u32(st, d_err, 1, 0u);
    launch_check_graph(st, n, ctx->d_rowptr, ctx->d_col, nnz, d_err);
    int err = 0;
    HIPCHK(d2h(ctx, &err, d_err, 1));
    static const char* const kWhy[] = {"", "a column index is out of range", "self loop",
                                       "columns of a row are not strictly ascending",
                                       "an edge is stored in one direction only"};
    NEED(err == 0, GCO_EINVAL, "malformed graph: %s", kWhy[err < 5 ? err : 0]);

    launch_fill_u32(st, d_count + n, 2, 0u);  // count[n] = 0
    launch_local_count(st, n, ctx->d_rowptr, ctx->d_col, ctx->d_part, ctx->d_perm, d_count);
    exclusive_scan_i64(st, d_count, d_lptr64, static_cast<int64_t>(n) + 1, d_scan);
    int64_t nnz_loc = 0;
    HIPCHK(d2h(ctx, &nnz_loc, d_lptr64 + n, 1));
    NEED(nnz_loc < std::numeric_limits<int32_t>::max(), GCO_ERANGE,
         "more than 2^31 local CSR entries");
    ctx->nnz_loc = nnz_loc;
    GALLOC(ctx->d_lrowptr, static_cast<size_t>(n) + 1);
    GALLOC(ctx->d_lcol, static_cast<size_t>(nnz_loc));
    launch_local_fill(st, n, ctx->d_rowptr, ctx->d_col, ctx->d_part, ctx->d_perm, ctx->d_inv,
                      d_lptr64, ctx->d_lrowptr, ctx->d_lcol);
    HIPCHK(d2h(ctx, lrowptr.data(), ctx->d_lrowptr, lrowptr.size()));
  }

  GALLOC(ctx->d_sa, static_cast<size_t>(n));
  GALLOC(ctx->d_sb, static_cast<size_t>(n));
  GALLOC(ctx->d_cbase, static_cast<size_t>(n));
  GALLOC(ctx->d_c, static_cast<size_t>(n));
  launch_scales(st, n, ctx->d_lrowptr, ctx->cfg.norm, ctx->cfg.problem, ctx->cfg.beta, ctx->d_sa,
                ctx->d_sb, ctx->d_cbase);
  launch_linear_coeff(st, n, ctx->d_cbase, nullptr, ctx->d_perm, ctx->d_c);
  // packed {column, A_hat value} entries of A_hat and of its transpose, and the diagonal
  // (the entry arrays carry kEntPad zero entries at the end: tiles copy a fixed number of
  // entries starting at their first one)
  GALLOC(ctx->d_ent, static_cast<size_t>(ctx->nnz_loc) + kEntPad);
  launch_fill_u32(st, ctx->d_ent + ctx->nnz_loc, 2 * kEntPad, 0u);
  GALLOC(ctx->d_diag, static_cast<size_t>(n));
  launch_pack_entries(st, n, ctx->d_lrowptr, ctx->d_lcol, ctx->d_sa, ctx->d_sb, ctx->d_ent, ctx->d_diag);
  if (ctx->cfg.norm == GCO_NORM_SYM) {
    ctx->d_ent_t = ctx->d_ent;  // symmetric normalisation: A_hat^T = A_hat
  } else {
    GALLOC(ctx->d_ent_t, static_cast<size_t>(ctx->nnz_loc) + kEntPad);
    launch_fill_u32(st, ctx->d_ent_t + ctx->nnz_loc, 2 * kEntPad, 0u);
    launch_pack_entries(st, n, ctx->d_lrowptr, ctx->d_lcol, ctx->d_sb, ctx->d_sa, ctx->d_ent_t, nullptr);
  }

  // light stream for the wave-per-tile kernels
  {
    Scratch tmp(ctx);
    int64_t* d_cnt = tmp.get<int64_t>(static_cast<size_t>(n) + 1);
    int64_t* d_wptr64 = tmp.get<int64_t>(static_cast<size_t>(n) + 1);
    int64_t* d_scan = tmp.get<int64_t>(scan_temp_elems(static_cast<int64_t>(n) + 1));
    NEED(d_cnt && d_wptr64 && d_scan, GCO_ENOMEM, "device scratch allocation failed");
    launch_fill_u32(st, d_cnt + n, 2, 0u);
    launch_light_count(st, n, ctx->d_lrowptr, d_cnt);
    exclusive_scan_i64(st, d_cnt, d_wptr64, static_cast<int64_t>(n) + 1, d_scan);
    int64_t nnz_light = 0;
    HIPCHK(d2h(ctx, &nnz_light, d_wptr64 + n, 1));
    NEED(nnz_light + kEntPad < std::numeric_limits<int32_t>::max(), GCO_ERANGE,
         "nodes plus local entries exceed 32-bit offsets");
    GALLOC(ctx->d_wrowptr, static_cast<size_t>(n) + 1);
    GALLOC(ctx->d_went, static_cast<size_t>(nnz_light) + kEntPad);
    launch_fill_u32(st, ctx->d_went + nnz_light, 2 * kEntPad, 0u);
    GALLOC(ctx->d_wval, static_cast<size_t>(nnz_light) + kEntPad);
    launch_fill_u32(st, ctx->d_wval + nnz_light, kEntPad, 0u);
    GALLOC(ctx->d_wrowid, static_cast<size_t>(nnz_light) + kEntPad);
    launch_fill_u32(st, ctx->d_wrowid + nnz_light, kEntPad, 0xffffffffu);
    launch_light_fill(st, n, ctx->d_lrowptr, ctx->d_ent, ctx->d_diag, d_wptr64, ctx->d_wrowptr, ctx->d_went,
                      ctx->d_wval, ctx->d_wrowid);
    if (ctx->d_ent_t == ctx->d_ent) {
      ctx->d_went_t = ctx->d_went;
      ctx->d_wval_t = ctx->d_wval;
    } else {
      GALLOC(ctx->d_wval_t, static_cast<size_t>(nnz_light) + kEntPad);
      launch_fill_u32(st, ctx->d_wval_t + nnz_light, kEntPad, 0u);
      GALLOC(ctx->d_went_t, static_cast<size_t>(nnz_light) + kEntPad);
      launch_fill_u32(st, ctx->d_went_t + nnz_light, 2 * kEntPad, 0u);
      launch_light_fill(st, n, ctx->d_lrowptr, ctx->d_ent_t, ctx->d_diag, d_wptr64, ctx->d_wrowptr,
                        ctx->d_went_t, ctx->d_wval_t, nullptr);
    }
  }

  // work decomposition
  std::vector<int> blk_k, blk_s, blk_S, nblk_k, nblk_s, nblk_S;
  // subgraph -> XCD affinity only when one feature matrix exceeds the 256 MB Infinity Cache
  const bool group_by_xcd =
      static_cast<double>(n) * ctx->cfg.dim * ctx->elem_bytes() > 256.0 * 1024 * 1024;
  build_block_map(P, part_rows, lrowptr, kTileRows, kWideBlocks, kMaxTilesPerBlock, blk_k, blk_s, blk_S,
                  group_by_xcd);
  // one decomposition per kernel kind (different cost per row)
  for (int v = 0; v < kWaveMaps; ++v) {
    std::vector<WaveRun> wave_runs;
    build_wave_map(P, part_rows, lrowptr, (ctx->cfg.dim == 128 ? kWaveBlocksFor128 : kWaveBlocksFor)[v],
                   kWaveRowCost[v], group_by_xcd, ctx->hm.wblk_k[v],
                   wave_runs);
    ctx->num_wblocks[v] = static_cast<int>(ctx->hm.wblk_k[v].size());
    GALLOC(ctx->d_wave_runs[v], wave_runs.size());
    HIPCHK(h2d(ctx, ctx->d_wave_runs[v], wave_runs.data(), wave_runs.size()));
  }
  // width-1 kernels: one 256-row tile per workgroup
  build_block_map(P, part_rows, lrowptr, kNarrowRows, std::numeric_limits<int>::max() / 2, 1, nblk_k,
                  nblk_s, nblk_S, group_by_xcd);
  GALLOC(ctx->d_blk_s, blk_s.size());
  GALLOC(ctx->d_nblk_s, nblk_s.size());
  GALLOC(ctx->d_blk_S, blk_S.size());
  GALLOC(ctx->d_nblk_S, nblk_S.size());
  HIPCHK(h2d(ctx, ctx->d_blk_S, blk_S.data(), blk_S.size()));
  HIPCHK(h2d(ctx, ctx->d_nblk_S, nblk_S.data(), nblk_S.size()));
  HIPCHK(h2d(ctx, ctx->d_blk_s, blk_s.data(), blk_s.size()));
  HIPCHK(h2d(ctx, ctx->d_nblk_s, nblk_s.data(), nblk_s.size()));
  ctx->hm.blk_k = blk_k;
  ctx->hm.nblk_k = nblk_k;
  // very long rows
  std::vector<int> heavy_of_row, heavy_rows, heavy_chunk_ptr(1, 0), chunk_begin, chunk_end, chunk_part;
  int num_heavy = 0;
  {
    int k = 0;
    for (int r = 0; r < n; ++r) {
      while (r >= part_rows[k + 1]) ++k;
      const int deg = lrowptr[r + 1] - lrowptr[r];
      if (deg >= kHeavyMin) {
        if (heavy_of_row.empty()) heavy_of_row.assign(n, -1);
        heavy_of_row[r] = num_heavy++;
        heavy_rows.push_back(r);
        for (int e = lrowptr[r]; e < lrowptr[r + 1]; e += kChunk) {
          chunk_begin.push_back(e);
          chunk_end.push_back(std::min(e + kChunk, lrowptr[r + 1]));
          chunk_part.push_back(k);
        }
        heavy_chunk_ptr.push_back(static_cast<int>(chunk_begin.size()));
      }
    }
  }
  const int num_chunks = static_cast<int>(chunk_begin.size());
  {  // subgraph of every pre-reduced row
    ctx->hm.heavy_part.clear();
    int kk = 0;
    for (int r : heavy_rows) {
      while (r >= part_rows[kk + 1]) ++kk;
      ctx->hm.heavy_part.push_back(kk);
    }
    ctx->hm.heavy_rows = heavy_rows;
    ctx->hm.chunk_part = chunk_part;
    ctx->num_loss_slots = static_cast<int>(heavy_rows.size() + ctx->hm.wblk_k[WM_NARROW].size());
  }
  {  // Form of the scalar layer's three passes.
     // ONE launch (a workgroup per subgraph, vectors in LDS): if two vectors of the largest
     // subgraph fit a compute unit's LDS and no subgraph is so large that its one workgroup
     // would take longer than three launches spread over the whole chip (measured at c4: one
     // subgraph with 147 k entries of the light stream, 3.8 times the mean, 0.40 ms against
     // 0.09 ms).  Else three launches that STAGE the gathered vector of a subgraph in LDS
     // (several workgroups per subgraph), if that vector fits twice per compute unit.  Else
     // three launches that gather from memory.
    int max_rows = 0;
    int64_t max_light = 0, total_light = 0;
    std::vector<int64_t> light_of(P, 0);
    for (int kk = 0; kk < P; ++kk) {
      max_rows = std::max(max_rows, part_rows[kk + 1] - part_rows[kk]);
      int64_t light = 0;
      for (int r = part_rows[kk]; r < part_rows[kk + 1]; ++r) {
        const int deg = lrowptr[r + 1] - lrowptr[r];
        light += 1 + (deg >= kHeavyMin ? 0 : deg);
      }
      light_of[kk] = light;
      total_light += light;
      max_light = std::max(max_light, light);
    }
    const int cap = std::max(4, (max_rows + 3) / 4 * 4);
    constexpr size_t kLdsPerComputeUnit = 160 * 1024;
    constexpr int64_t kFusedMaxEntries = 40960;  // 40 steps per wavefront and pass
    const int fused_nw = max_rows > 2048 ? 16 : 4;
    const bool fused_fits = scalar_fused_lds_bytes(fused_nw, cap) <= kLdsPerComputeUnit;
    const int staged_cap = (max_rows + 3 + 3) / 4 * 4;
    const bool staged_fits =
        2 * scalar_staged_lds_bytes(staged_cap) <= kLdsPerComputeUnit && staged_cap <= scalar_staged_max_cap();
    const int form = ctx->scalar_form_wanted;
    NEED(form != GCO_SCALAR_ONE_LAUNCH || fused_fits, GCO_ERANGE,
         "the one-launch scalar layer needs two vectors of the largest subgraph (%d rows) in %zu bytes of LDS",
         max_rows, kLdsPerComputeUnit);
    NEED(form != GCO_SCALAR_STAGED || staged_fits, GCO_ERANGE,
         "the staged scalar layer needs the largest subgraph's vector (%d rows) twice in %zu bytes of LDS and at "
         "most %d rows", max_rows, kLdsPerComputeUnit, scalar_staged_max_cap() - 3);
    ctx->fused_scalar =
        form == GCO_SCALAR_ONE_LAUNCH || (form == GCO_SCALAR_AUTO && fused_fits && max_light <= kFusedMaxEntries);
    ctx->staged_scalar = form == GCO_SCALAR_STAGED || (form == GCO_SCALAR_AUTO && !ctx->fused_scalar && staged_fits);
    ctx->fused_waves = fused_nw;
    ctx->fused_cap = cap;
    ctx->staged_cap = staged_cap;
    ctx->hm.staged_k.clear();
    if (ctx->fused_scalar || ctx->staged_scalar) {
      // workgroups per subgraph: one, or (staged) a share of about two per compute unit in
      // proportion to the subgraph's entries, such that a wavefront keeps a few steps of work
      const int NW = ctx->fused_scalar ? fused_nw : scalar_staged_waves();
      std::vector<int> wg_ptr(static_cast<size_t>(P) + 1, 0);
      const int64_t target = std::max<int64_t>(P, std::min<int64_t>(512, total_light / (static_cast<int64_t>(NW) * 256)));
      std::vector<int> per_part(static_cast<size_t>(P), 1);
      if (ctx->staged_scalar && total_light > 0) {
        std::vector<double> work(light_of.begin(), light_of.end());
        per_part = apportion(work, target, std::vector<int>(static_cast<size_t>(P), 1),
                             std::vector<int>(static_cast<size_t>(P), static_cast<int>(target)));
      }
      for (int kk = 0; kk < P; ++kk) {
        const int per = per_part[kk];
        wg_ptr[kk + 1] = wg_ptr[kk] + per;
        for (int q = 0; q < per; ++q) ctx->hm.staged_k.push_back(kk);
      }
      const int num_wgs = wg_ptr[P];
      ctx->num_loss_slots = num_wgs;
      // Launch order of the staged form: workgroup ids go round the 8 XCDs, so the
      // workgroups of a subgraph get ids that are equal mod 8: they share one L2, and the
      // vector they all copy is fetched into it once.  Subgraphs are dealt to the XCD with
      // the least work so far; launch_of[b] = workgroup that launch id b stands for (-1: none).
      std::vector<int> launch_of;
      if (ctx->staged_scalar) {
        std::vector<std::vector<int>> on_xcd(8);
        for (int kk = 0; kk < P; ++kk) {
          size_t best = 0;
          for (size_t x = 1; x < 8; ++x)
            if (on_xcd[x].size() < on_xcd[best].size()) best = x;
          for (int w = wg_ptr[kk]; w < wg_ptr[kk + 1]; ++w) on_xcd[best].push_back(w);
        }
        size_t depth = 0;
        for (const auto& v : on_xcd) depth = std::max(depth, v.size());
        launch_of.assign(depth * 8, -1);
        for (size_t x = 0; x < 8; ++x)
          for (size_t q = 0; q < on_xcd[x].size(); ++q) launch_of[q * 8 + x] = on_xcd[x][q];
      }
      ctx->staged_wgs = static_cast<int>(launch_of.size());
      // rows of every subgraph cut into contiguous runs of about equal cost (entries of the
      // light stream plus one per row), one per wavefront of its workgroups; a run is handed
      // over as its range of the stream
      std::vector<int2> cuts(static_cast<size_t>(num_wgs) * NW);
      int64_t woff = 0;  // light-stream offset of the current row
      for (int kk = 0; kk < P; ++kk) {
        const int rb = part_rows[kk], re = part_rows[kk + 1];
        const int V = (wg_ptr[kk + 1] - wg_ptr[kk]) * NW;
        std::vector<double> pre(static_cast<size_t>(re - rb) + 1, 0.0);
        std::vector<int> off(static_cast<size_t>(re - rb) + 1, 0);
        for (int r = rb; r < re; ++r) {
          const int deg = lrowptr[r + 1] - lrowptr[r];
          const int len = 1 + (deg >= kHeavyMin ? 0 : deg);
          off[r - rb] = static_cast<int>(woff);
          woff += len;
          pre[r - rb + 1] = pre[r - rb] + 1 + len;
        }
        off[re - rb] = static_cast<int>(woff);
        int r = rb;
        for (int v = 0; v < V; ++v) {
          const int start = r;
          const double want = pre[re - rb] * (v + 1) / V;
          while (r < re && (v == V - 1 || pre[r - rb + 1] <= want)) ++r;
          cuts[static_cast<size_t>(wg_ptr[kk]) * NW + v] = make_int2(off[start - rb], off[r - rb]);
        }
      }
      std::vector<int> heavy_ptr(static_cast<size_t>(P) + 1, 0);
      for (int kk : ctx->hm.heavy_part) heavy_ptr[kk + 1]++;
      for (int kk = 0; kk < P; ++kk) heavy_ptr[kk + 1] += heavy_ptr[kk];
      GALLOC(ctx->d_fused_cuts, cuts.size());
      GALLOC(ctx->d_heavy_ptr, heavy_ptr.size());
      GALLOC(ctx->d_staged_k, ctx->hm.staged_k.size());
      GALLOC(ctx->d_staged_ptr, wg_ptr.size());
      if (!launch_of.empty()) {
        GALLOC(ctx->d_staged_launch, launch_of.size());
        HIPCHK(h2d(ctx, ctx->d_staged_launch, launch_of.data(), launch_of.size()));
      }
      HIPCHK(h2d(ctx, ctx->d_fused_cuts, cuts.data(), cuts.size()));
      HIPCHK(h2d(ctx, ctx->d_heavy_ptr, heavy_ptr.data(), heavy_ptr.size()));
      HIPCHK(h2d(ctx, ctx->d_staged_k, ctx->hm.staged_k.data(), ctx->hm.staged_k.size()));
      HIPCHK(h2d(ctx, ctx->d_staged_ptr, wg_ptr.data(), wg_ptr.size()));
    }
  }
  ctx->full.allocated = false;
  ctx->sub.allocated = false;
  {
    const int rc = upload_active_maps(ctx, ctx->full, nullptr);
    if (rc != GCO_OK) return rc;
  }
  {  // pre-reduced rows per wave tile
    std::vector<int> tbase(P + 1, 0);
    for (int kk = 0; kk < P; ++kk)
      tbase[kk + 1] = tbase[kk] + (part_rows[kk + 1] - part_rows[kk] + kWaveRows - 1) / kWaveRows;
    std::vector<int> hptr(static_cast<size_t>(tbase[P]) + 1, 0);
    int kk = 0;
    for (int r : heavy_rows) {
      while (r >= part_rows[kk + 1]) ++kk;
      hptr[tbase[kk] + (r - part_rows[kk]) / kWaveRows + 1]++;
    }
    for (size_t q = 1; q < hptr.size(); ++q) hptr[q] += hptr[q - 1];
    GALLOC(ctx->d_wtile_hptr, hptr.size());
    HIPCHK(h2d(ctx, ctx->d_wtile_hptr, hptr.data(), hptr.size()));
  }
  if (num_heavy > 0) {
    GALLOC(ctx->d_heavy_of_row, static_cast<size_t>(n));
    GALLOC(ctx->d_heavy_chunk_ptr, heavy_chunk_ptr.size());
    GALLOC(ctx->d_chunk_begin, chunk_begin.size());
    GALLOC(ctx->d_chunk_end, chunk_end.size());
    GALLOC(ctx->d_heavy_partial, static_cast<size_t>(num_chunks) * D);
    GALLOC(ctx->d_heavy_partial_E, static_cast<size_t>(num_chunks) * D);
    HIPCHK(h2d(ctx, ctx->d_heavy_of_row, heavy_of_row.data(), heavy_of_row.size()));
    HIPCHK(h2d(ctx, ctx->d_heavy_chunk_ptr, heavy_chunk_ptr.data(), heavy_chunk_ptr.size()));
    HIPCHK(h2d(ctx, ctx->d_chunk_begin, chunk_begin.data(), chunk_begin.size()));
    HIPCHK(h2d(ctx, ctx->d_chunk_end, chunk_end.data(), chunk_end.size()));
    // parts of the pre-reduced rows for the width-1 launches
    std::vector<int2> hpart;
    std::vector<int> hpart_ptr(1, 0);
    for (int hh = 0; hh < num_heavy; ++hh) {
      const int chunks = heavy_chunk_ptr[hh + 1] - heavy_chunk_ptr[hh];
      const int parts = (chunks + kNarrowPartChunks - 1) / kNarrowPartChunks;
      for (int j = 0; j < parts; ++j) hpart.push_back(make_int2(hh, j));
      hpart_ptr.push_back(static_cast<int>(hpart.size()));
    }
    ctx->num_hparts = static_cast<int>(hpart.size());
    const std::vector<int> zeros(static_cast<size_t>(num_heavy), 0);
    GALLOC(ctx->d_hpart, hpart.size());
    GALLOC(ctx->d_hpart_ptr, hpart_ptr.size());
    GALLOC(ctx->d_hpart_partial, hpart.size());
    GALLOC(ctx->d_hpart_count, zeros.size());
    HIPCHK(h2d(ctx, ctx->d_hpart, hpart.data(), hpart.size()));
    HIPCHK(h2d(ctx, ctx->d_hpart_ptr, hpart_ptr.data(), hpart_ptr.size()));
    HIPCHK(h2d(ctx, ctx->d_hpart_count, zeros.data(), zeros.size()));
  }

  GraphView& g = ctx->gv;
  g = GraphView{};
  g.n = n;
  g.P = P;
  g.rowptr = ctx->d_lrowptr;
  g.col = ctx->d_lcol;
  g.sa = ctx->d_sa;
  g.sb = ctx->d_sb;
  g.part_rows = ctx->d_part_rows;
  g.blk_k = ctx->full.blk_k;
  g.blk_s = ctx->d_blk_s;
  g.blk_S = ctx->d_blk_S;
  g.num_blocks = static_cast<int>(blk_k.size());
  for (int v = 0; v < kWaveMaps; ++v) {
    g.wave_runs[v] = ctx->d_wave_runs[v];
    g.wblk_k[v] = ctx->full.wblk_k[v];
    g.num_wblocks[v] = ctx->num_wblocks[v];
  }
  g.wrowptr = ctx->d_wrowptr;
  g.wtile_hptr = ctx->d_wtile_hptr;
  g.went = ctx->d_went;
  g.went_t = ctx->d_went_t;
  g.wval = ctx->d_wval;
  g.wval_t = ctx->d_wval_t;
  g.wrowid = ctx->d_wrowid;
  g.nblk_k = ctx->full.nblk_k;
  g.nblk_s = ctx->d_nblk_s;
  g.nblk_S = ctx->d_nblk_S;
  g.num_nblocks = static_cast<int>(nblk_k.size());
  g.num_loss_slots = ctx->num_loss_slots;
  g.loss_ptr = ctx->full.loss_ptr;
  g.loss_list = ctx->full.loss_list;
  g.num_heavy = num_heavy;
  g.num_chunks = num_chunks;
  g.heavy_of_row = ctx->d_heavy_of_row;
  g.heavy_rows = ctx->full.heavy_rows;
  g.ent = ctx->d_ent;
  g.ent_t = ctx->d_ent_t;
  g.diag = ctx->d_diag;
  g.heavy_chunk_ptr = ctx->d_heavy_chunk_ptr;
  g.chunk_begin = ctx->d_chunk_begin;
  g.chunk_end = ctx->d_chunk_end;
  g.chunk_part = ctx->full.chunk_part;
  g.num_hparts = ctx->num_hparts;
  g.hpart = ctx->d_hpart;
  g.hpart_ptr = ctx->d_hpart_ptr;
  g.hpart_partial = ctx->d_hpart_partial;
  g.hpart_count = ctx->d_hpart_count;

  // parameters, optimizer state, activations
  const size_t nd = static_cast<size_t>(n) * D;
  const int eb = ctx->elem_bytes();
  GALLOC(ctx->E, nd);
  GALLOC(ctx->mE, nd);
  GALLOC(ctx->vE, nd);
  if (eb == 2) {
    uint16_t* q = nullptr;
    GALLOC(q, nd);
    ctx->Eb = q;
    ctx->H[0] = q;
  } else {
    ctx->Eb = nullptr;
    ctx->H[0] = ctx->E;
  }
  for (int l = 1; l <= L; ++l) {
    const size_t cnt = static_cast<size_t>(ctx->Pw) * w_elems(ctx, l);
    GALLOC(ctx->W[l - 1], cnt);
    GALLOC(ctx->mW[l - 1], cnt);
    GALLOC(ctx->vW[l - 1], cnt);
  }
  for (int l = 1; l <= L - 1; ++l) {
    uint8_t* q = nullptr;
    GALLOC(q, nd * eb);
    ctx->H[l] = q;
    GALLOC(ctx->gW_partial[l - 1],
           static_cast<size_t>(std::max({g.num_blocks, g.num_wblocks[WM_BWD], g.num_wblocks[WM_EMBED], g.num_wblocks[WM_GRADW]})) * D * D);
  }
  // G_Z between two hidden layers; the wave-per-tile kernels also store that of the last one
  for (int l = 1; l <= (ctx->wave_path() ? L - 1 : L - 2); ++l) {
    uint8_t* q = nullptr;
    GALLOC(q, nd * eb);
    ctx->GZ[l] = q;
  }
  if (ctx->split_grad_w() && L >= 2) {
    uint8_t* q = nullptr;
    GALLOC(q, nd * eb);
    ctx->GT = q;
  }
  GALLOC(ctx->gwout_partial, static_cast<size_t>(std::max(g.num_blocks, g.num_nblocks)) * D);
  GALLOC(ctx->d_bc, static_cast<size_t>(kLossSets) * (P + ctx->Pw));
  GALLOC(ctx->t, static_cast<size_t>(n));
  GALLOC(ctx->z, static_cast<size_t>(n));
  GALLOC(ctx->p, static_cast<size_t>(n));
  GALLOC(ctx->g_z, static_cast<size_t>(n));
  GALLOC(ctx->g_t, static_cast<size_t>(n));
  GALLOC(ctx->loss_partial, static_cast<size_t>(g.num_loss_slots) * kLossSets);
  GALLOC(ctx->loss_part, static_cast<size_t>(P));
  GALLOC(ctx->loss_one, 1);
  HIPCHK(hipStreamSynchronize(st));
  traffic_model(ctx);
  ctx->has_graph = true;
  ctx->stepE.assign(static_cast<size_t>(ctx->P), 0);
  ctx->stepW.assign(static_cast<size_t>(ctx->Pw), 0);
  return GCO_OK;
}

int gco_graph_info(gco_ctx* ctx, int64_t* n, int64_t* m, int64_t* m_local, int64_t* m_cut) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_graph, GCO_ESTATE, "no graph uploaded");
  if (n) *n = ctx->n;
  if (m) *m = ctx->nnz_full / 2;
  if (m_local) *m_local = ctx->nnz_loc / 2;
  if (m_cut) *m_cut = (ctx->nnz_full - ctx->nnz_loc) / 2;
  return GCO_OK;
}

// ---- parameter transfer -------------------------------------------------------

static int upload_node_matrix(gco_ctx* ctx, const float* host_orig, float* dev_new) {
  const size_t nd = static_cast<size_t>(ctx->n) * ctx->cfg.dim;
  Scratch tmp(ctx);
  float* stage = tmp.get<float>(nd);
  NEED(stage, GCO_ENOMEM, "device scratch allocation failed");
  HIPCHK(h2d(ctx, stage, host_orig, nd));
  launch_gather_rows(ctx->st, ctx->n, ctx->cfg.dim, stage, ctx->d_perm, dev_new);
  return GCO_OK;
}

static int download_node_matrix(gco_ctx* ctx, float* host_orig, const float* dev_new) {
  const size_t nd = static_cast<size_t>(ctx->n) * ctx->cfg.dim;
  Scratch tmp(ctx);
  float* stage = tmp.get<float>(nd);
  NEED(stage, GCO_ENOMEM, "device scratch allocation failed");
  launch_gather_rows(ctx->st, ctx->n, ctx->cfg.dim, dev_new, ctx->d_inv, stage);
  HIPCHK(d2h(ctx, host_orig, stage, nd));
  return GCO_OK;
}

// Forget every snapshot: lowest loss +infinity, no model has one.
static int reset_best(gco_ctx* ctx) {
  const std::vector<double> inf(static_cast<size_t>(ctx->Pw), std::numeric_limits<double>::infinity());
  HIPCHK(h2d(ctx, ctx->d_best_loss, inf.data(), inf.size()));
  HIPCHK(hipMemsetAsync(ctx->d_has_best, 0, static_cast<size_t>(ctx->Pw) * sizeof(int32_t), ctx->st));
  HIPCHK(hipMemsetAsync(ctx->d_improved, 0, static_cast<size_t>(ctx->Pw) * sizeof(int32_t), ctx->st));
  return GCO_OK;
}

// Parameters from the host; with U != nullptr the embeddings pass through the
// Gumbel-softmax of Sec. 3.2 first.
static int set_params_impl(gco_ctx* ctx, const float* E, const float* U, float tau, const float* const* W) {
  NEED(ctx->has_graph, GCO_ESTATE, "no graph uploaded");
  NEED(E && W, GCO_EINVAL, "NULL parameter pointer");
  const int L = ctx->cfg.num_layers;
  for (int l = 1; l <= L; ++l) NEED(W[l - 1], GCO_EINVAL, "W[%d] is NULL", l - 1);
  const size_t nd = static_cast<size_t>(ctx->n) * ctx->cfg.dim;
  int rc = upload_node_matrix(ctx, E, ctx->E);
  if (rc != GCO_OK) return rc;
  if (U != nullptr) {
    Scratch tmp(ctx);
    float* d_u = tmp.get<float>(nd);
    NEED(d_u, GCO_ENOMEM, "device scratch allocation failed");
    rc = upload_node_matrix(ctx, U, d_u);
    if (rc != GCO_OK) return rc;
    launch_gumbel_softmax_rows(ctx->launch(), ctx->n, ctx->cfg.dim, ctx->E, d_u, tau);
    HIPCHK(hipStreamSynchronize(ctx->st));  // d_u is released on return
  }
  HIPCHK(hipMemsetAsync(ctx->mE, 0, nd * sizeof(float), ctx->st));
  HIPCHK(hipMemsetAsync(ctx->vE, 0, nd * sizeof(float), ctx->st));
  for (int l = 1; l <= L; ++l) {
    const size_t cnt = static_cast<size_t>(ctx->Pw) * w_elems(ctx, l);
    HIPCHK(h2d(ctx, ctx->W[l - 1], W[l - 1], cnt));
    HIPCHK(hipMemsetAsync(ctx->mW[l - 1], 0, cnt * sizeof(float), ctx->st));
    HIPCHK(hipMemsetAsync(ctx->vW[l - 1], 0, cnt * sizeof(float), ctx->st));
  }
  if (ctx->Eb) launch_to_bf16(ctx->launch(), ctx->E, ctx->Eb, static_cast<int64_t>(nd));
  ctx->heavy_E_valid = false;
  if (ctx->best_alloc) {
    rc = reset_best(ctx);
    if (rc != GCO_OK) return rc;
  }
  HIPCHK(hipStreamSynchronize(ctx->st));
  ctx->stepE.assign(static_cast<size_t>(ctx->P), 0);
  ctx->stepW.assign(static_cast<size_t>(ctx->Pw), 0);
  ctx->has_params = true;
  ctx->probs_valid = false;
  return GCO_OK;
}

int gco_set_params(gco_ctx* ctx, const float* E, const float* const* W) {
  if (!ctx) return GCO_EINVAL;
  return set_params_impl(ctx, E, nullptr, 1.f, W);
}

int gco_set_params_gumbel(gco_ctx* ctx, const float* E, const float* U, float tau, const float* const* W) {
  if (!ctx) return GCO_EINVAL;
  NEED(U, GCO_EINVAL, "U is NULL");
  NEED(tau > 0.f, GCO_EINVAL, "tau must be positive");
  return set_params_impl(ctx, E, U, tau, W);
}

int gco_get_params(gco_ctx* ctx, float* E, float* const* W) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_params, GCO_ESTATE, "no parameters set");
  if (E) {
    int rc = download_node_matrix(ctx, E, ctx->E);
    if (rc != GCO_OK) return rc;
  }
  if (W)
    for (int l = 1; l <= ctx->cfg.num_layers; ++l)
      if (W[l - 1])
        HIPCHK(d2h(ctx, W[l - 1], ctx->W[l - 1], static_cast<size_t>(ctx->Pw) * w_elems(ctx, l)));
  return GCO_OK;
}

int gco_get_opt_state(gco_ctx* ctx, float* mE, float* vE, float* const* mW, float* const* vW,
                      int64_t* step) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_params, GCO_ESTATE, "no parameters set");
  int rc;
  if (mE && (rc = download_node_matrix(ctx, mE, ctx->mE)) != GCO_OK) return rc;
  if (vE && (rc = download_node_matrix(ctx, vE, ctx->vE)) != GCO_OK) return rc;
  for (int l = 1; l <= ctx->cfg.num_layers; ++l) {
    const size_t cnt = static_cast<size_t>(ctx->Pw) * w_elems(ctx, l);
    if (mW && mW[l - 1]) HIPCHK(d2h(ctx, mW[l - 1], ctx->mW[l - 1], cnt));
    if (vW && vW[l - 1]) HIPCHK(d2h(ctx, vW[l - 1], ctx->vW[l - 1], cnt));
  }
  if (step) {  // the largest count; gco_get_steps gives all of them
    *step = 0;
    for (int64_t t : ctx->stepE) *step = std::max(*step, t);
    for (int64_t t : ctx->stepW) *step = std::max(*step, t);
  }
  return GCO_OK;
}

int gco_set_opt_state(gco_ctx* ctx, const float* mE, const float* vE, const float* const* mW,
                      const float* const* vW, int64_t step) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_params, GCO_ESTATE, "no parameters set");
  NEED(mE && vE && mW && vW && step >= 0, GCO_EINVAL, "bad optimizer state argument");
  int rc;
  if ((rc = upload_node_matrix(ctx, mE, ctx->mE)) != GCO_OK) return rc;
  if ((rc = upload_node_matrix(ctx, vE, ctx->vE)) != GCO_OK) return rc;
  for (int l = 1; l <= ctx->cfg.num_layers; ++l) {
    NEED(mW[l - 1] && vW[l - 1], GCO_EINVAL, "NULL moment pointer for layer %d", l);
    const size_t cnt = static_cast<size_t>(ctx->Pw) * w_elems(ctx, l);
    HIPCHK(h2d(ctx, ctx->mW[l - 1], mW[l - 1], cnt));
    HIPCHK(h2d(ctx, ctx->vW[l - 1], vW[l - 1], cnt));
  }
  HIPCHK(hipStreamSynchronize(ctx->st));
  ctx->stepE.assign(static_cast<size_t>(ctx->P), step);
  ctx->stepW.assign(static_cast<size_t>(ctx->Pw), step);
  return GCO_OK;
}

int gco_set_linear_penalty(gco_ctx* ctx, const float* extra) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_graph, GCO_ESTATE, "no graph uploaded");
  if (!extra) {
    launch_linear_coeff(ctx->st, ctx->n, ctx->d_cbase, nullptr, ctx->d_perm, ctx->d_c);
    return GCO_OK;
  }
  Scratch tmp(ctx);
  float* stage = tmp.get<float>(static_cast<size_t>(ctx->n));
  NEED(stage, GCO_ENOMEM, "device scratch allocation failed");
  HIPCHK(h2d(ctx, stage, extra, static_cast<size_t>(ctx->n)));
  launch_linear_coeff(ctx->st, ctx->n, ctx->d_cbase, stage, ctx->d_perm, ctx->d_c);
  return GCO_OK;
}

// ---- one epoch ------------------------------------------------------------------

// Hidden layers of Eq. 3 and the transform of the scalar layer: leaves t.
static void run_hidden_forward(gco_ctx* ctx, const GraphView& gv) {
  const Launch ln = ctx->launch();
  const gco_config& c = ctx->cfg;
  const int D = c.dim, L = c.num_layers;
  const int ws = ctx->Pw == 1 ? 0 : D * D, wos = ctx->Pw == 1 ? 0 : D;
  if (L == 1) {
    launch_fwd_gemv(ln, c.storage, D, gv, ctx->H[0], ctx->W[0], wos, ctx->t);
  } else {
    for (int l = 1; l <= L - 1; ++l) {
      const bool last = l == L - 1;
      const bool ready = l == 1 && ctx->heavy_E_valid && ctx->d_heavy_partial_E != nullptr;
      launch_fwd_hidden(ln, c.storage, D, gv, ctx->H[l - 1], ctx->W[l - 1], ws, ctx->H[l],
                        last ? ctx->W[L - 1] : nullptr, wos, ctx->t,
                        ready ? ctx->d_heavy_partial_E : ctx->d_heavy_partial, ready);
    }
  }
}

// The width-1 passes on t: passes = 1: z = A_hat t, p = sigmoid(z) (Eq. 4); 2: also the
// loss partials of set `slot` (< kLossSets) and dL/dz (Eq. 5); 3: also g_t = A_hat^T dL/dz.
// One launch when the subgraphs fit a compute unit's LDS, else one launch per pass.
static void run_scalar_layer(gco_ctx* ctx, const GraphView& gv, int passes, int slot) {
  const Launch ln = ctx->launch();
  const float q = ctx->cfg.problem == GCO_PROBLEM_MAXCUT ? 2.f : ctx->cfg.alpha;
  double* partial = ctx->loss_partial + static_cast<size_t>(slot) * gv.num_loss_slots;
  if (ctx->fused_scalar) {
    launch_scalar_fused(ln, gv, ctx->fused_waves, ctx->fused_cap, ctx->d_fused_cuts, ctx->d_heavy_ptr, ctx->t,
                        ctx->p, ctx->d_c, q, ctx->g_t, partial, passes);
  } else {
    ScalarStaging staging;
    staging.num_launch = ctx->staged_wgs;
    staging.cap = ctx->staged_cap;
    staging.cuts = ctx->d_fused_cuts;
    staging.heavy_ptr = ctx->d_heavy_ptr;
    staging.wg_k = ctx->d_staged_k;
    staging.wg_ptr = ctx->d_staged_ptr;
    staging.launch_of = ctx->d_staged_launch;
    const ScalarStaging* sg = ctx->staged_scalar ? &staging : nullptr;
    launch_fwd_readout(ln, gv, ctx->t, ctx->z, ctx->p, sg);
    if (passes >= 2) launch_loss(ln, gv, ctx->p, ctx->d_c, q, ctx->g_z, partial, sg);
    if (passes >= 3) launch_bwd_readout(ln, gv, ctx->g_z, ctx->g_t, sg);
  }
  ctx->probs_valid = true;
}

static void run_forward(gco_ctx* ctx) {
  run_hidden_forward(ctx, ctx->gv);
  run_scalar_layer(ctx, ctx->gv, 1, 0);
}

// Adam constants for one more step when every subgraph and weight set has seen `step` steps.
static AdamStep adam_constants(const gco_config& c, int64_t step) {
  AdamStep ad{};
  const double tt = static_cast<double>(step);
  ad.lr = c.lr;
  ad.b1 = c.adam_b1;
  ad.b2 = c.adam_b2;
  ad.eps = c.adam_eps;
  ad.inv_bc1 = static_cast<float>(1.0 / (1.0 - std::pow(static_cast<double>(c.adam_b1), tt)));
  ad.inv_sqrt_bc2 = static_cast<float>(1.0 / std::sqrt(1.0 - std::pow(static_cast<double>(c.adam_b2), tt)));
  return ad;
}

// Backward pass from g_t on (run_scalar_layer with passes = 3 has run).
// update = true: an Adam step with the constants adE (embedding rows) and adW (weights);
// update = false: gradients are written to gE / gW.  gv and maps name the subgraphs that
// take part.
static void run_backward(gco_ctx* ctx, const GraphView& gv, const gco_ctx::ActiveMaps& maps, bool update,
                         const AdamStep& adE, const AdamStep& adW, float* gE, float* const* gW) {
  const Launch ln = ctx->launch();
  const gco_config& c = ctx->cfg;
  const int D = c.dim, L = c.num_layers;
  const int ws = ctx->Pw == 1 ? 0 : D * D, wos = ctx->Pw == 1 ? 0 : D;
  const AdamStep& ad = adE;
  BwdArgs a;
  a.g_t = ctx->g_t;
  a.w_out = ctx->W[L - 1];
  a.wout_stride = wos;
  a.gwout_partial = ctx->gwout_partial;
  a.E = ctx->E;
  a.mE = ctx->mE;
  a.vE = ctx->vE;
  a.Eb = ctx->Eb;
  a.gE = gE;
  a.adam = ad;
  a.heavy_partial = ctx->d_heavy_partial;
  a.GZ_last = L >= 2 ? ctx->GZ[L - 1] : nullptr;
  a.GT = ctx->GT;
  a.mode = update ? (c.train_embed ? EMBED_ADAM : EMBED_SKIP) : (gE ? EMBED_WRITE_GRAD : EMBED_SKIP);
  if (L == 1) {
    a.Hprev = ctx->H[0];
    launch_bwd_single(ln, c.storage, D, gv, a);
  } else {
    for (int l = L - 1; l >= 1; --l) {
      const bool last = l == L - 1, to_embed = l == 1;
      a.GZ_in = last ? nullptr : ctx->GZ[l];
      a.Hcur = last ? ctx->H[l] : nullptr;
      a.Hprev = ctx->H[l - 1];
      a.W = ctx->W[l - 1];
      a.w_stride = ws;
      a.gW_partial = ctx->gW_partial[l - 1];
      a.GZ_out = to_embed ? nullptr : ctx->GZ[l - 1];
      launch_bwd_hidden(ln, c.storage, D, last, to_embed, gv, a);
    }
  }
  WeightTensor wt[3];
  for (int l = 1; l <= L; ++l) {
    wt[l - 1].W = ctx->W[l - 1];
    wt[l - 1].m = ctx->mW[l - 1];
    wt[l - 1].v = ctx->vW[l - 1];
    wt[l - 1].partial = l < L ? ctx->gW_partial[l - 1] : ctx->gwout_partial;
    wt[l - 1].grad_out = (!update && gW) ? gW[l - 1] : nullptr;
    wt[l - 1].elems = w_elems(ctx, l);
    // who wrote the partials: the wide kernels' workgroups, or, on the wave-per-tile path,
    // its own workgroups (hidden layers) and the narrow ones (scalar layer)
    const bool wave = ctx->wave_path() && L >= 2;
    const int wm = ctx->grad_map(l);  // the decomposition whose workgroups wrote gW_l
    wt[l - 1].blk_ptr = !wave ? maps.pbl_ptr : (l < L ? maps.wpbl_ptr[wm] : maps.nwbl_ptr);
    wt[l - 1].blk_list = !wave ? maps.pbl_list : (l < L ? maps.wpbl_list[wm] : maps.nwbl_list);
  }
  const int writers = (ctx->wave_path() && L >= 2)
                          ? std::max({gv.num_wblocks[WM_BWD], gv.num_wblocks[WM_EMBED], gv.num_nblocks})
                          : gv.num_blocks;
  const bool many_partials = writers / ctx->Pw >= 512;
  // the last launch of an epoch also pre-reduces the long rows of the new embeddings
  ChunkTail tail;
  const bool fold = update && c.train_embed && ctx->wave_path() && L >= 2 && gv.num_chunks > 0 && !many_partials;
  if (fold) {
    tail.g = gv;
    tail.X = ctx->Eb;
    tail.partial = ctx->d_heavy_partial_E;
    tail.D = D;
  }
  if (update && c.train_embed && !fold) ctx->heavy_E_valid = false;  // the embeddings change, the partials do not follow
  launch_adam_w(ln, ctx->Pw, wt, L, adW, update, many_partials, fold ? &tail : nullptr);
  // a run over a subset refreshes only its own subgraphs' chunks: valid only on top of valid
  if (fold) ctx->heavy_E_valid = ctx->heavy_E_valid || &maps == &ctx->full;
  if (update) ctx->probs_valid = true;  // p is that of the parameters before the step
}

// Copies the parameters of the models flagged on the device between the live set and the
// snapshot.
static void copy_params(gco_ctx* ctx, const GraphView& gv, const int32_t* flag, bool to_best) {
  const int L = ctx->cfg.num_layers;
  int elems[3] = {};
  for (int l = 1; l <= L; ++l) elems[l - 1] = static_cast<int>(w_elems(ctx, l));
  if (to_best)
    launch_param_copy(ctx->launch(), gv, ctx->Pw, ctx->cfg.dim, flag, ctx->E, ctx->E_best, ctx->W,
                      ctx->W_best, elems, L);
  else
    launch_param_copy(ctx->launch(), gv, ctx->Pw, ctx->cfg.dim, flag, ctx->E_best, ctx->E, ctx->W_best,
                      ctx->W, elems, L);
}

// `epochs` training epochs of the subgraphs with active[k] != 0 (nullptr: all of them); the
// others keep their parameters, optimizer state, step counts and probabilities.
static int train_impl(gco_ctx* ctx, int32_t epochs, const uint8_t* active, double* loss_per_epoch) {
  const int P = ctx->P, Pw = ctx->Pw;
  const GraphView& gv = active ? ctx->gv_sub : ctx->gv;
  const gco_ctx::ActiveMaps& maps = active ? ctx->sub : ctx->full;
  if (ctx->loss_hist_cap < epochs) {
    // grow geometrically; the old array is released once the stream has drained
    if (ctx->loss_hist != nullptr) {
      HIPCHK(hipStreamSynchronize(ctx->st));
      auto it = std::find(ctx->graph_allocs.begin(), ctx->graph_allocs.end(), static_cast<void*>(ctx->loss_hist));
      if (it != ctx->graph_allocs.end()) ctx->graph_allocs.erase(it);
      ctx->raw_free(ctx->loss_hist);
      ctx->loss_hist = nullptr;
      ctx->loss_hist_cap = 0;
    }
    const int64_t cap = std::max<int64_t>(epochs, 2 * ctx->loss_hist_cap);
    GALLOC(ctx->loss_hist, static_cast<size_t>(cap));
    ctx->loss_hist_cap = cap;
  }
  // which weight sets take part: a subgraph's own, or the shared one if any subgraph does
  std::vector<uint8_t> actE(P, 1), actW(Pw, 0);
  if (active) actE.assign(active, active + P);
  for (int k = 0; k < P; ++k)
    if (actE[k]) actW[Pw == 1 ? 0 : k] = 1;
  // one set of Adam constants serves all while every step count is the same
  bool uniform = active == nullptr;
  for (int64_t t : ctx->stepE) uniform = uniform && t == ctx->stepE[0];
  for (int64_t t : ctx->stepW) uniform = uniform && t == ctx->stepE[0];
  const gco_config& c = ctx->cfg;
  std::vector<float2> bc;
  // the loss partials of up to kLossSets epochs are reduced by one launch; so are the
  // per-subgraph bias corrections of those epochs uploaded at once
  for (int e0 = 0; e0 < epochs; e0 += kLossSets) {
    const int ne = std::min<int>(kLossSets, epochs - e0);
    if (!uniform) {
      bc.assign(static_cast<size_t>(ne) * (P + Pw), make_float2(1.f, 1.f));
      for (int e = 0; e < ne; ++e)
        for (int q = 0; q < P + Pw; ++q) {
          const bool on = q < P ? actE[q] : actW[q - P];
          if (!on) continue;
          const int64_t t0 = q < P ? ctx->stepE[q] : ctx->stepW[q - P];
          const AdamStep ad = adam_constants(c, t0 + e0 + e + 1);
          bc[static_cast<size_t>(e) * (P + Pw) + q] = make_float2(ad.inv_bc1, ad.inv_sqrt_bc2);
        }
      HIPCHK(h2d(ctx, ctx->d_bc, bc.data(), bc.size()));
    }
    for (int e = 0; e < ne; ++e) {
      AdamStep adE = adam_constants(c, ctx->stepE.empty() ? 1 : ctx->stepE[0] + e0 + e + 1), adW = adE;
      if (!uniform) {
        adE.per_part = ctx->d_bc + static_cast<size_t>(e) * (P + Pw);
        adW.per_part = adE.per_part + P;
      }
      run_hidden_forward(ctx, gv);
      run_scalar_layer(ctx, gv, 3, e);
      if (ctx->best_on) {
        // the parameters still are the ones this loss belongs to
        launch_best_update(ctx->launch(), gv, ctx->loss_partial + static_cast<size_t>(e) * gv.num_loss_slots,
                           Pw, ctx->d_best_loss, ctx->d_improved, ctx->d_has_best);
        copy_params(ctx, gv, ctx->d_improved, /*to_best=*/true);
      }
      run_backward(ctx, gv, maps, true, adE, adW, nullptr, nullptr);
    }
    launch_loss_reduce(ctx->launch(), gv, ctx->loss_partial, ne, gv.num_loss_slots, nullptr, ctx->loss_hist + e0);
  }
  for (int k = 0; k < P; ++k)
    if (actE[k]) ctx->stepE[k] += epochs;
  for (int k = 0; k < Pw; ++k)
    if (actW[k]) ctx->stepW[k] += epochs;
  HIPCHK(hipGetLastError());
  if (loss_per_epoch) HIPCHK(d2h(ctx, loss_per_epoch, ctx->loss_hist, static_cast<size_t>(epochs)));
  return GCO_OK;
}

int gco_train(gco_ctx* ctx, int32_t epochs, double* loss_per_epoch) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_params, GCO_ESTATE, "set_params must precede train");
  NEED(epochs >= 0, GCO_EINVAL, "negative epoch count");
  if (epochs == 0) return GCO_OK;
  return train_impl(ctx, epochs, nullptr, loss_per_epoch);
}

int gco_train_subset(gco_ctx* ctx, int32_t epochs, const int32_t* parts, int32_t num_listed,
                     double* loss_per_epoch) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_params, GCO_ESTATE, "set_params must precede train");
  NEED(epochs >= 0, GCO_EINVAL, "negative epoch count");
  NEED(num_listed >= 0 && (parts != nullptr || num_listed == 0), GCO_EINVAL, "bad subgraph list");
  std::vector<uint8_t> active(static_cast<size_t>(ctx->P), 0);
  for (int q = 0; q < num_listed; ++q) {
    NEED(parts[q] >= 0 && parts[q] < ctx->P, GCO_ERANGE, "subgraph id %d out of range", parts[q]);
    active[parts[q]] = 1;
  }
  if (epochs == 0 || num_listed == 0) {
    if (loss_per_epoch)
      for (int e = 0; e < epochs; ++e) loss_per_epoch[e] = 0.0;
    return GCO_OK;
  }
  // the maps of the previous call serve again when the same subgraphs are listed (the
  // fine-tuning rounds of Alg. 1 stage 3 come back with the same set many times)
  if (!ctx->sub.allocated || ctx->sub_active != active) {
    const int rc = upload_active_maps(ctx, ctx->sub, active.data());
    if (rc != GCO_OK) return rc;
    ctx->sub_active = active;
  }
  ctx->gv_sub = view_with(ctx, ctx->sub);
  return train_impl(ctx, epochs, active.data(), loss_per_epoch);
}

int gco_keep_best(gco_ctx* ctx, int32_t enable) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_graph, GCO_ESTATE, "no graph uploaded");
  if (!enable) {
    ctx->best_on = false;
    return GCO_OK;
  }
  if (!ctx->best_alloc) {
    GALLOC(ctx->E_best, static_cast<size_t>(ctx->n) * ctx->cfg.dim);
    for (int l = 1; l <= ctx->cfg.num_layers; ++l)
      GALLOC(ctx->W_best[l - 1], static_cast<size_t>(ctx->Pw) * w_elems(ctx, l));
    GALLOC(ctx->d_best_loss, static_cast<size_t>(ctx->Pw));
    GALLOC(ctx->d_improved, static_cast<size_t>(ctx->Pw));
    GALLOC(ctx->d_has_best, static_cast<size_t>(ctx->Pw));
    ctx->best_alloc = true;
  }
  const int rc = reset_best(ctx);
  if (rc != GCO_OK) return rc;
  HIPCHK(hipStreamSynchronize(ctx->st));
  ctx->best_on = true;
  return GCO_OK;
}

int gco_get_best_loss(gco_ctx* ctx, double* best_loss) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->best_alloc, GCO_ESTATE, "gco_keep_best was never enabled");
  NEED(best_loss, GCO_EINVAL, "best_loss is NULL");
  HIPCHK(d2h(ctx, best_loss, ctx->d_best_loss, static_cast<size_t>(ctx->Pw)));
  return GCO_OK;
}

int gco_restore_best(gco_ctx* ctx) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->best_alloc, GCO_ESTATE, "gco_keep_best was never enabled");
  NEED(ctx->has_params, GCO_ESTATE, "no parameters set");
  copy_params(ctx, ctx->gv, ctx->d_has_best, /*to_best=*/false);
  if (ctx->Eb)
    launch_to_bf16(ctx->launch(), ctx->E, ctx->Eb, static_cast<int64_t>(ctx->n) * ctx->cfg.dim);
  ctx->heavy_E_valid = false;
  HIPCHK(hipGetLastError());
  ctx->probs_valid = false;
  return GCO_OK;
}

int gco_get_steps(gco_ctx* ctx, int64_t* steps_embed, int64_t* steps_weights) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_params, GCO_ESTATE, "set_params must precede get_steps");
  if (steps_embed) std::copy(ctx->stepE.begin(), ctx->stepE.end(), steps_embed);
  if (steps_weights) std::copy(ctx->stepW.begin(), ctx->stepW.end(), steps_weights);
  return GCO_OK;
}

int gco_set_steps(gco_ctx* ctx, const int64_t* steps_embed, const int64_t* steps_weights) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_params, GCO_ESTATE, "set_params must precede set_steps");
  NEED(steps_embed && steps_weights, GCO_EINVAL, "NULL step array");
  for (int k = 0; k < ctx->P; ++k) NEED(steps_embed[k] >= 0, GCO_EINVAL, "negative step count");
  for (int k = 0; k < ctx->Pw; ++k) NEED(steps_weights[k] >= 0, GCO_EINVAL, "negative step count");
  ctx->stepE.assign(steps_embed, steps_embed + ctx->P);
  ctx->stepW.assign(steps_weights, steps_weights + ctx->Pw);
  return GCO_OK;
}

int gco_forward(gco_ctx* ctx) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_params, GCO_ESTATE, "set_params must precede forward");
  run_forward(ctx);
  HIPCHK(hipGetLastError());
  return GCO_OK;
}

int gco_get_probs(gco_ctx* ctx, float* p) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->probs_valid, GCO_ESTATE, "no forward pass has run");
  NEED(p, GCO_EINVAL, "p is NULL");
  Scratch tmp(ctx);
  float* stage = tmp.get<float>(static_cast<size_t>(ctx->n));
  NEED(stage, GCO_ENOMEM, "device scratch allocation failed");
  launch_gather_rows(ctx->st, ctx->n, 1, ctx->p, ctx->d_inv, stage);
  HIPCHK(d2h(ctx, p, stage, static_cast<size_t>(ctx->n)));
  return GCO_OK;
}

int gco_loss(gco_ctx* ctx, double* total, double* per_part) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_params, GCO_ESTATE, "set_params must precede loss");
  run_hidden_forward(ctx, ctx->gv);
  run_scalar_layer(ctx, ctx->gv, 2, 0);
  launch_loss_reduce(ctx->launch(), ctx->gv, ctx->loss_partial, 1, 0, ctx->loss_part, ctx->loss_one);
  HIPCHK(hipGetLastError());
  if (total) HIPCHK(d2h(ctx, total, ctx->loss_one, 1));
  if (per_part) HIPCHK(d2h(ctx, per_part, ctx->loss_part, static_cast<size_t>(ctx->P)));
  return GCO_OK;
}

int gco_get_grads(gco_ctx* ctx, float* gE, float* const* gW) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_params, GCO_ESTATE, "set_params must precede get_grads");
  const int L = ctx->cfg.num_layers;
  const size_t nd = static_cast<size_t>(ctx->n) * ctx->cfg.dim;
  Scratch tmp(ctx);
  float* d_gE = gE ? tmp.get<float>(nd) : nullptr;
  NEED(!gE || d_gE, GCO_ENOMEM, "device scratch allocation failed");
  float* d_gW[3] = {};
  for (int l = 1; l <= L; ++l) {
    d_gW[l - 1] = tmp.get<float>(static_cast<size_t>(ctx->Pw) * w_elems(ctx, l));
    NEED(d_gW[l - 1], GCO_ENOMEM, "device scratch allocation failed");
  }
  run_hidden_forward(ctx, ctx->gv);
  run_scalar_layer(ctx, ctx->gv, 3, 0);
  run_backward(ctx, ctx->gv, ctx->full, false, AdamStep{}, AdamStep{}, d_gE, d_gW);
  HIPCHK(hipGetLastError());
  if (gE) {
    int rc = download_node_matrix(ctx, gE, d_gE);
    if (rc != GCO_OK) return rc;
  }
  if (gW)
    for (int l = 1; l <= L; ++l)
      if (gW[l - 1])
        HIPCHK(d2h(ctx, gW[l - 1], d_gW[l - 1], static_cast<size_t>(ctx->Pw) * w_elems(ctx, l)));
  return GCO_OK;
}

int gco_get_hidden(gco_ctx* ctx, int32_t layer, float* H) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->probs_valid, GCO_ESTATE, "no forward pass has run");
  NEED(H, GCO_EINVAL, "H is NULL");
  NEED(layer >= 1 && layer <= ctx->cfg.num_layers - 1, GCO_EINVAL, "layer %d has no hidden activation", layer);
  const size_t nd = static_cast<size_t>(ctx->n) * ctx->cfg.dim;
  const float* src = static_cast<const float*>(ctx->H[layer]);
  Scratch tmp(ctx);
  if (ctx->cfg.storage == GCO_STORAGE_BF16) {
    float* wide = tmp.get<float>(nd);
    NEED(wide, GCO_ENOMEM, "device scratch allocation failed");
    launch_from_bf16(ctx->launch(), ctx->H[layer], wide, static_cast<int64_t>(nd));
    src = wide;
  }
  return download_node_matrix(ctx, H, src);
}

// ---- read-out -------------------------------------------------------------------

// Device buffers of one gco_round_repair call (n floats, three byte arrays of n rounded up
// to a multiple of 4, 8 counters, 4 ints).
struct RepairBuffers {
  float* p_orig;
  uint8_t *state, *x_orig, *x_new;
  unsigned long long* counts;
  int* undecided;
};

static int round_repair_impl(gco_ctx* ctx, float thr, int32_t repair_scope, const RepairBuffers& b, uint8_t* x,
                             int64_t* objective, int64_t* conflicts_before, int64_t* conflicts_after) {
  const int n = ctx->n;
  hipStream_t st = ctx->st;
  float* p_orig = b.p_orig;
  uint8_t *state = b.state, *x_orig = b.x_orig, *x_new = b.x_new;
  unsigned long long* counts = b.counts;
  int* undecided = b.undecided;
  launch_gather_rows(st, n, 1, ctx->p, ctx->d_inv, p_orig);
  launch_round(st, n, p_orig, thr, x_orig);  // 0/1 in original order
  launch_fill_u32(st, counts, 16, 0u);
  launch_edge_counts(st, n, ctx->d_rowptr, ctx->d_col, x_orig, counts);
  const bool repair = ctx->cfg.problem == GCO_PROBLEM_MIS && repair_scope != GCO_REPAIR_NONE;
  if (repair) {
    const bool local = repair_scope == GCO_REPAIR_LOCAL;
    if (local) launch_round(st, n, ctx->p, thr, state);
    else launch_round(st, n, p_orig, thr, state);
    // each batch of four rounds ends with a count of the nodes still undecided
    for (int64_t guard = 0; guard <= static_cast<int64_t>(n) + 4; guard += 4) {
      launch_fill_u32(st, undecided, 4, 0u);
      for (int q = 0; q < 4; ++q) {
        if (local)
          launch_repair_round_local(st, n, ctx->d_lrowptr, ctx->d_lcol, ctx->p, state, undecided + q);
        else
          launch_repair_round_all(st, n, ctx->d_rowptr, ctx->d_col, p_orig, state, undecided + q);
      }
      int left = 0;
      HIPCHK(d2h(ctx, &left, undecided + 3, 1));
      if (left == 0) break;
    }
    if (local) {
      launch_state_to_x(st, n, state, x_new);
      launch_gather_bytes(st, n, x_new, ctx->d_inv, x_orig);
    } else {
      launch_state_to_x(st, n, state, x_orig);
    }
  }
  launch_edge_counts(st, n, ctx->d_rowptr, ctx->d_col, x_orig, counts + 4);
  unsigned long long h[8];
  HIPCHK(d2h(ctx, h, counts, 8));
  HIPCHK(d2h(ctx, x, x_orig, static_cast<size_t>(n)));
  if (conflicts_before) *conflicts_before = static_cast<int64_t>(h[1]);
  if (conflicts_after) *conflicts_after = static_cast<int64_t>(h[5]);
  if (objective)
    *objective = static_cast<int64_t>(ctx->cfg.problem == GCO_PROBLEM_MIS ? h[4] : h[6]);
  return GCO_OK;
}

int gco_round_repair(gco_ctx* ctx, float thr, int32_t repair_scope, uint8_t* x, int64_t* objective,
                     int64_t* conflicts_before, int64_t* conflicts_after) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->probs_valid, GCO_ESTATE, "no forward pass has run");
  NEED(x, GCO_EINVAL, "x is NULL");
  NEED(repair_scope >= GCO_REPAIR_NONE && repair_scope <= GCO_REPAIR_ALL, GCO_EINVAL,
       "bad repair_scope %d", repair_scope);
  const int n = ctx->n;
  Scratch tmp(ctx);
  const size_t npad = (static_cast<size_t>(n) + 3) / 4 * 4;
  RepairBuffers b{};
  b.p_orig = tmp.get<float>(static_cast<size_t>(n));
  b.state = tmp.get<uint8_t>(npad);
  b.x_orig = tmp.get<uint8_t>(npad);
  b.x_new = tmp.get<uint8_t>(npad);
  b.counts = tmp.get<unsigned long long>(8);
  b.undecided = tmp.get<int>(4);
  NEED(b.p_orig && b.state && b.x_orig && b.x_new && b.counts && b.undecided, GCO_ENOMEM,
       "device scratch allocation failed");
  return round_repair_impl(ctx, thr, repair_scope, b, x, objective, conflicts_before, conflicts_after);
}

int gco_round_repair_static(gco_ctx* ctx, float thr, int32_t repair_scope, uint8_t* x, int64_t* objective,
                            int64_t* conflicts_before, int64_t* conflicts_after) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->probs_valid, GCO_ESTATE, "no forward pass has run");
  NEED(x, GCO_EINVAL, "x is NULL");
  NEED(repair_scope >= GCO_REPAIR_NONE && repair_scope <= GCO_REPAIR_ALL, GCO_EINVAL,
       "bad repair_scope %d", repair_scope);
  NEED(ctx->n <= kStaticMaxNodes, GCO_ERANGE,
       "n = %d exceeds the %d nodes the static work area of gco_round_repair_static holds", ctx->n,
       kStaticMaxNodes);
  void* base = nullptr;
  HIPCHK(static_scratch_for_current_device(&base));
  // carve the block: every piece starts on a 256-byte boundary
  const size_t n = static_cast<size_t>(ctx->n);
  const size_t npad = (n + 3) / 4 * 4;
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  unsigned char* q = static_cast<unsigned char*>(base);
  RepairBuffers b{};
  b.counts = reinterpret_cast<unsigned long long*>(q);
  q += 256;
  b.undecided = reinterpret_cast<int*>(q);
  q += 256;
  b.p_orig = reinterpret_cast<float*>(q);
  q += up(n * sizeof(float));
  b.state = q;
  q += up(npad);
  b.x_orig = q;
  q += up(npad);
  b.x_new = q;
  q += up(npad);
  NEED(static_cast<size_t>(q - static_cast<unsigned char*>(base)) <= kStaticScratchBytes, GCO_ERANGE,
       "static work area too small for n = %d", ctx->n);
  return round_repair_impl(ctx, thr, repair_scope, b, x, objective, conflicts_before, conflicts_after);
}

static int cross_edges_impl(gco_ctx* ctx, const uint8_t* d_x, int64_t* count, int32_t* u, int32_t* v,
                            uint8_t* cross_host) {
  const int n = ctx->n;
  hipStream_t st = ctx->st;
  Scratch tmp(ctx);
  int64_t* cnt = tmp.get<int64_t>(static_cast<size_t>(n) + 1);
  int64_t* offs = tmp.get<int64_t>(static_cast<size_t>(n) + 1);
  int64_t* scan = tmp.get<int64_t>(scan_temp_elems(static_cast<int64_t>(n) + 1));
  NEED(cnt && offs && scan, GCO_ENOMEM, "device scratch allocation failed");
  launch_fill_u32(st, cnt + n, 2, 0u);
  launch_cut_count(st, n, ctx->d_rowptr, ctx->d_col, ctx->d_part, d_x, cnt);
  exclusive_scan_i64(st, cnt, offs, static_cast<int64_t>(n) + 1, scan);
  int64_t total = 0;
  HIPCHK(d2h(ctx, &total, offs + n, 1));
  if (cross_host) {
    const size_t npad = (static_cast<size_t>(n) + 3) / 4 * 4;
    uint8_t* cross = tmp.get<uint8_t>(npad);
    NEED(cross, GCO_ENOMEM, "device scratch allocation failed");
    launch_fill_u32(st, cross, static_cast<int64_t>(npad / 4), 0u);
    launch_cut_fill(st, n, ctx->d_rowptr, ctx->d_col, ctx->d_part, d_x, offs, nullptr, nullptr, cross);
    HIPCHK(d2h(ctx, cross_host, cross, static_cast<size_t>(n)));
    return GCO_OK;
  }
  if (!u && !v) {
    *count = total;
    return GCO_OK;
  }
  NEED(u && v, GCO_EINVAL, "u and v must both be given");
  NEED(*count >= total, GCO_ERANGE, "capacity %lld < %lld cross edges",
       static_cast<long long>(*count), static_cast<long long>(total));
  int32_t* du = tmp.get<int32_t>(static_cast<size_t>(total));
  int32_t* dv = tmp.get<int32_t>(static_cast<size_t>(total));
  NEED(du && dv, GCO_ENOMEM, "device scratch allocation failed");
  launch_cut_fill(st, n, ctx->d_rowptr, ctx->d_col, ctx->d_part, d_x, offs, du, dv, nullptr);
  HIPCHK(d2h(ctx, u, du, static_cast<size_t>(total)));
  HIPCHK(d2h(ctx, v, dv, static_cast<size_t>(total)));
  *count = total;
  return GCO_OK;
}

int gco_cut_edges(gco_ctx* ctx, int64_t* count, int32_t* u, int32_t* v) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_graph, GCO_ESTATE, "no graph uploaded");
  NEED(count, GCO_EINVAL, "count is NULL");
  return cross_edges_impl(ctx, nullptr, count, u, v, nullptr);
}

int gco_cross_mask(gco_ctx* ctx, uint8_t* c) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_graph, GCO_ESTATE, "no graph uploaded");
  NEED(c, GCO_EINVAL, "c is NULL");
  int64_t dummy = 0;
  return cross_edges_impl(ctx, nullptr, &dummy, nullptr, nullptr, c);
}

int gco_conflict_edges(gco_ctx* ctx, const uint8_t* x, int64_t* count, int32_t* u, int32_t* v) {
  if (!ctx) return GCO_EINVAL;
  NEED(ctx->has_graph, GCO_ESTATE, "no graph uploaded");
  NEED(x && count, GCO_EINVAL, "x or count is NULL");
  Scratch tmp(ctx);
  uint8_t* dx = tmp.get<uint8_t>(static_cast<size_t>(ctx->n));
  NEED(dx, GCO_ENOMEM, "device scratch allocation failed");
  HIPCHK(h2d(ctx, dx, x, static_cast<size_t>(ctx->n)));
  return cross_edges_impl(ctx, dx, count, u, v, nullptr);
}

// ---- timing ---------------------------------------------------------------------

int gco_set_profiling(gco_ctx* ctx, int32_t mode, uint64_t kind_mask) {
  if (!ctx) return GCO_EINVAL;
  NEED(mode >= 0 && mode <= 3, GCO_EINVAL, "bad profiling mode %d", mode);
  HIPCHK(hipStreamSynchronize(ctx->st));
  ctx->prof.harvest();
  ctx->prof.mode = mode;
  ctx->prof.mask = kind_mask;
  for (int k = 0; k < KK_COUNT; ++k) ctx->prof.seen[k] = 0;
  return GCO_OK;
}

int gco_apportion(const double* work, int32_t n, int64_t target, const int32_t* lo, const int32_t* hi,
                  int32_t* share) {
  if (!work || !lo || !hi || !share || n < 0 || target < 0) return GCO_EINVAL;
  for (int k = 0; k < n; ++k)
    if (lo[k] < 0 || lo[k] > hi[k] || !(work[k] >= 0.0)) return GCO_EINVAL;
  const std::vector<int> got = apportion(std::vector<double>(work, work + n), target, std::vector<int>(lo, lo + n),
                                         std::vector<int>(hi, hi + n));
  std::copy(got.begin(), got.end(), share);
  return GCO_OK;
}

int gco_num_kernel_kinds(void) { return KK_COUNT; }

const char* gco_kernel_kind_name(int32_t kind) {
  return kind >= 0 && kind < KK_COUNT ? kKindNames[kind] : "";
}

int gco_get_timing(gco_ctx* ctx, int32_t kind, int64_t* launches, double* total_ms,
                   double* algorithmic_bytes_per_launch) {
  if (!ctx) return GCO_EINVAL;
  NEED(kind >= 0 && kind < KK_COUNT, GCO_EINVAL, "bad kernel kind %d", kind);
  HIPCHK(hipStreamSynchronize(ctx->st));
  ctx->prof.harvest();
  if (launches) *launches = ctx->prof.launches[kind];
  if (total_ms) *total_ms = ctx->prof.total_ms[kind];
  if (algorithmic_bytes_per_launch) *algorithmic_bytes_per_launch = ctx->kind_bytes[kind];
  return GCO_OK;
}

int gco_reset_timing(gco_ctx* ctx) {
  if (!ctx) return GCO_EINVAL;
  HIPCHK(hipStreamSynchronize(ctx->st));
  ctx->prof.reset();
  return GCO_OK;
}

}  // extern "C"
