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
//
// The gather is organised to keep many loads in flight, because its address
// chain (row pointer -> entry -> feature row) is otherwise paid serially:
//   * the row pointers of every tile a workgroup owns are read into LDS once;
//   * CSR entries are packed as {column, scale} pairs; the entries and the own
//     rows of tile q+1 are requested before tile q is gathered and parked in
//     registers, then committed to LDS when tile q is done;
//   * a lane group gathers its rows of the tile together, eight 16-byte row
//     slices per lane in flight, and sums them in a fixed order.
#include <type_traits>

#include "bf16_common.h"
#include "device_utils.h"
#include "gco_internal.h"

namespace gco {
namespace {


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
  static constexpr int G = kBlock / LPR;                // lane groups per workgroup
  static constexpr int NCH = R / G;                     // rows of a tile per lane group
  static constexpr int UNR = 8 / NCH;                   // entries per row requested together
  static_assert(NCH >= 1 && NCH * G == R && UNR >= 1, "tile rows must divide over the lane groups");
  static constexpr int PO = D + 4;                      // pitch of the fp32 staging tile
  static constexpr size_t at_bytes = static_cast<size_t>(R) * PA * 2;
  static constexpr size_t tt_bytes = static_cast<size_t>(D) * PT * 2;
  static_assert(at_bytes % 16 == 0 && tt_bytes % 16 == 0, "tile alignment");
  static_assert(at_bytes + tt_bytes >= static_cast<size_t>(R) * PO * 4, "fp32 staging must fit");
};



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

constexpr int kEntCap = 512;                 // CSR entries of a tile kept in LDS
constexpr int kEntPerThread = kEntCap / kBlock;


// Gather sources.  A source names the feature matrix whose rows are gathered,
// the scale of the own row (self loop) and of an entry, and how a raw 16-byte
// slice is added to the accumulator.
template <int D>
struct PlainB {  // acc += scale * X[j, c0..c0+8)
  const bf16_t* X;
  const float* diag;  // A_hat_ii
  __device__ __forceinline__ void set_part(int, int) {}
  __device__ __forceinline__ float own_scale(int i) const { return diag[i]; }
  __device__ __forceinline__ float entry_scale(int, float w) const { return w; }
  __device__ __forceinline__ void apply(const uint4& raw, float sc, float (&acc)[8]) const {
    float v[8];
    unpack8(raw, v);
#pragma unroll
    for (int x = 0; x < 8; ++x) acc[x] = fmaf(sc, v[x], acc[x]);
  }
};

template <int D>
struct LastB {  // gradient of the last hidden pre-activation, formed on the fly:
                // acc += scale * g_t[j] * w_out[c] * [H[j, c] > 0]
  const bf16_t* X;
  const float* diag;  // A_hat_ii
  const float* g_t;
  const float* w_out;
  int wout_stride;
  float w[8];
  __device__ __forceinline__ void set_part(int k, int c0) {
#pragma unroll
    for (int x = 0; x < 8; ++x) w[x] = w_out[static_cast<size_t>(k) * wout_stride + c0 + x];
  }
  __device__ __forceinline__ float own_scale(int i) const { return diag[i] * g_t[i]; }
  __device__ __forceinline__ float entry_scale(int j, float we) const { return we * g_t[j]; }
  __device__ __forceinline__ void apply(const uint4& raw, float sc, float (&acc)[8]) const {
    float v[8];
    unpack8(raw, v);
#pragma unroll
    for (int x = 0; x < 8; ++x) acc[x] += v[x] > 0.f ? sc * w[x] : 0.f;
  }
};

// What a thread holds of the next tile while the current one is worked on.
template <int D>
struct TileRegs {
  uint4 own[MG<D>::NCH];        // its slices of the tile's own rows (zero beyond the last row)
  int2 ent[kEntPerThread];      // its share of the tile's CSR entries
  bool in_lds;                  // the tile's entries fit the LDS buffer
};

template <int D, class Src>
__device__ __forceinline__ void prefetch_tile(const GraphView& g, const Src& src, int row0, int nrows,
                                              const int* rpq, TileRegs<D>& tr) {
  using M = MG<D>;
  const int tid = threadIdx.x;
  const int grp = tid / M::LPR, c0 = (tid % M::LPR) * 8;
#pragma unroll
  for (int u = 0; u < M::NCH; ++u) {
    const int r = grp + M::G * u;
    tr.own[u] = make_uint4(0u, 0u, 0u, 0u);
    if (r < nrows)
      tr.own[u] = *reinterpret_cast<const uint4*>(src.X + static_cast<size_t>(row0 + r) * D + c0);
  }
  const int e_base = rpq[0], E = rpq[R] - e_base;
  tr.in_lds = E <= kEntCap;
#pragma unroll
  for (int x = 0; x < kEntPerThread; ++x) {
    const int idx = tid + kBlock * x;
    tr.ent[x] = make_int2(0, 0);
    if (tr.in_lds && idx < E) tr.ent[x] = g.ent[e_base + idx];
  }
}

// out[u] = this thread's 16-byte slice of row row0 + grp + G * u of `base` (zero past nrows).
template <int D>
__device__ __forceinline__ void prefetch_rows(const bf16_t* base, int row0, int nrows,
                                              uint4 (&out)[MG<D>::NCH]) {
  using M = MG<D>;
  const int grp = threadIdx.x / M::LPR, c0 = (threadIdx.x % M::LPR) * 8;
#pragma unroll
  for (int u = 0; u < M::NCH; ++u) {
    const int r = grp + M::G * u;
    out[u] = make_uint4(0u, 0u, 0u, 0u);
    if (r < nrows) out[u] = *reinterpret_cast<const uint4*>(base + static_cast<size_t>(row0 + r) * D + c0);
  }
}

template <int D>
__device__ __forceinline__ void commit_entries(const TileRegs<D>& tr, int2* ents) {
  if (tr.in_lds) {
#pragma unroll
    for (int x = 0; x < kEntPerThread; ++x) ents[threadIdx.x + kBlock * x] = tr.ent[x];
  }
}


// Rows row0 .. row0+nrows of A_hat times the source matrix, into `sink`
// (rows nrows..R get zeros).  `rpq` holds the tile's R + 1 row pointers (LDS),
// `ents` the tile's entries if in_lds, `own` the thread's slices of the own rows.
// hlist[0] must be 0 on entry.  Ends with a barrier.
template <int D, class Src, class Sink>
__device__ void gather_tile(const GraphView& g, const Src& src, const Sink& sink, int row0, int nrows,
                            const int* rpq, const int2* ents, bool in_lds,
                            const uint4 (&own)[MG<D>::NCH], float* red, int* hlist,
                            const float* __restrict__ heavy_partial) {
  using M = MG<D>;
  const int tid = threadIdx.x;
  const int grp = tid / M::LPR, c0 = (tid % M::LPR) * 8;
  const int e_base = rpq[0];
  const auto entry = [&](int e) -> int2 { return in_lds ? ents[e - e_base] : g.ent[e]; };
  float acc[M::NCH][8];
  int pos[M::NCH], end[M::NCH];
  bool direct[M::NCH];  // this lane group finishes the row itself
#pragma unroll
  for (int u = 0; u < M::NCH; ++u) {
    const int r = grp + M::G * u;
#pragma unroll
    for (int x = 0; x < 8; ++x) acc[u][x] = 0.f;
    pos[u] = end[u] = 0;
    direct[u] = true;
    if (r < nrows) {
      const int i = row0 + r;
      const int ea = rpq[r], eb = rpq[r + 1];
      const int deg = eb - ea;
      if (deg >= kHeavyMin) {          // pre-reduced in chunks
        src.apply(own[u], src.own_scale(i), acc[u]);
        const int h = find_heavy(g, i);
        for (int ch = g.heavy_chunk_ptr[h]; ch < g.heavy_chunk_ptr[h + 1]; ++ch) {
          const float4* pp = reinterpret_cast<const float4*>(heavy_partial + static_cast<size_t>(ch) * D + c0);
          const float4 p0 = pp[0], p1 = pp[1];
          acc[u][0] += p0.x; acc[u][1] += p0.y; acc[u][2] += p0.z; acc[u][3] += p0.w;
          acc[u][4] += p1.x; acc[u][5] += p1.y; acc[u][6] += p1.z; acc[u][7] += p1.w;
        }
      } else if (deg > kLightMax) {    // left to the whole workgroup
        direct[u] = false;
        if (tid % M::LPR == 0) {
          const int q = atomicAdd(&hlist[0], 1);
          hlist[1 + q] = r;
        }
      } else {
        src.apply(own[u], src.own_scale(i), acc[u]);
        pos[u] = ea;
        end[u] = eb;
      }
    }
  }
  // rounds: UNR entries of each of the group's rows are requested together
  for (;;) {
    bool more = false;
#pragma unroll
    for (int u = 0; u < M::NCH; ++u) more = more || pos[u] < end[u];
    if (!more) break;
    uint4 raw[M::NCH][M::UNR];
    float sc[M::NCH][M::UNR];
#pragma unroll
    for (int u = 0; u < M::NCH; ++u) {
#pragma unroll
      for (int x = 0; x < M::UNR; ++x) {
        const int e = pos[u] + x;
        raw[u][x] = make_uint4(0u, 0u, 0u, 0u);
        sc[u][x] = 0.f;
        if (e < end[u]) {
          const int2 en = entry(e);
          raw[u][x] = *reinterpret_cast<const uint4*>(src.X + static_cast<size_t>(en.x) * D + c0);
          sc[u][x] = src.entry_scale(en.x, __int_as_float(en.y));
        }
      }
    }
#pragma unroll
    for (int u = 0; u < M::NCH; ++u) {
#pragma unroll
      for (int x = 0; x < M::UNR; ++x) src.apply(raw[u][x], sc[u][x], acc[u]);
      pos[u] += M::UNR;
    }
  }
#pragma unroll
  for (int u = 0; u < M::NCH; ++u) {
    const int r = grp + M::G * u;
    if (direct[u]) sink.template put_vec<8>(r, c0, acc[u]);
  }
  __syncthreads();
  const int nh = hlist[0];
  for (int q = 0; q < nh; ++q) {  // rows summed by all lane groups together
    const int r = hlist[1 + q];
    const int i = row0 + r;
    const int ea = rpq[r], eb = rpq[r + 1];
    float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (grp == 0) {
      const uint4 self = *reinterpret_cast<const uint4*>(src.X + static_cast<size_t>(i) * D + c0);
      src.apply(self, src.own_scale(i), a8);
    }
    for (int e = ea + grp; e < eb; e += 4 * M::G) {
      uint4 rw[4];
      float s4[4];
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        const int ee = e + x * M::G;
        rw[x] = make_uint4(0u, 0u, 0u, 0u);
        s4[x] = 0.f;
        if (ee < eb) {
          const int2 en = entry(ee);
          rw[x] = *reinterpret_cast<const uint4*>(src.X + static_cast<size_t>(en.x) * D + c0);
          s4[x] = src.entry_scale(en.x, __int_as_float(en.y));
        }
      }
#pragma unroll
      for (int x = 0; x < 4; ++x) src.apply(rw[x], s4[x], a8);
    }
#pragma unroll
    for (int x = 0; x < 8; ++x) red[grp * D + c0 + x] = a8[x];
    __syncthreads();
    if (tid < D) {
      float sum = 0.f;
      for (int gq = 0; gq < M::G; ++gq) sum += red[gq * D + tid];
      sink.put_one(r, tid, sum);
    }
    __syncthreads();
  }
}

// Chunked pre-reduction of very long rows: partial[c, :] = sum over the entries of chunk c.
template <int D, class Src>
__global__ __launch_bounds__(kBlock) void heavy_wide_b_kernel(GraphView g, Src src, float* partial) {
  using M = MG<D>;
  __shared__ float red[kBlock * 8];
  const int ch = blockIdx.x;
  const int tid = threadIdx.x;
  const int grp = tid / M::LPR, c0 = (tid % M::LPR) * 8;
  if (g.chunk_part[ch] < 0) return;  // the row's subgraph sits out
  src.set_part(g.chunk_part[ch], c0);
  float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const int eb = g.chunk_end[ch];
  for (int e = g.chunk_begin[ch] + grp; e < eb; e += 4 * M::G) {
    uint4 rw[4];
    float s4[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int ee = e + x * M::G;
      rw[x] = make_uint4(0u, 0u, 0u, 0u);
      s4[x] = 0.f;
      if (ee < eb) {
        const int2 en = g.ent[ee];
        rw[x] = *reinterpret_cast<const uint4*>(src.X + static_cast<size_t>(en.x) * D + c0);
        s4[x] = src.entry_scale(en.x, __int_as_float(en.y));
      }
    }
#pragma unroll
    for (int x = 0; x < 4; ++x) src.apply(rw[x], s4[x], a8);
  }
#pragma unroll
  for (int x = 0; x < 8; ++x) red[grp * D + c0 + x] = a8[x];
  __syncthreads();
  if (tid < D) {
    float sum = 0.f;
    for (int gq = 0; gq < M::G; ++gq) sum += red[gq * D + tid];
    partial[static_cast<size_t>(ch) * D + tid] = sum;
  }
}

// Row pointers of every tile this workgroup owns -> LDS: rp[q * (R + 1) + t] is
// the pointer of row min(row0_q + t, rend), so rows past the subgraph are empty.
__device__ __forceinline__ int preload_row_pointers(const GraphView& g, int rbeg, int rend, int s,
                                                    int S, int* rp) {
  const int tiles = (rend - rbeg + R - 1) / R;
  const int Q = tiles > s ? (tiles - s + S - 1) / S : 0;
  for (int idx = threadIdx.x; idx < Q * (R + 1); idx += kBlock) {
    const int q = idx / (R + 1), t = idx % (R + 1);
    rp[idx] = g.rowptr[min(rbeg + (s + q * S) * R + t, rend)];
  }
  return Q;
}

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

constexpr size_t kGatherLds = kBlock * 8 * sizeof(float)                      // red
                              + kEntCap * sizeof(int2)                        // ents
                              + kMaxTilesPerBlock * (R + 1) * sizeof(int)     // rp
                              + (R + 4) * sizeof(int);                        // hlist
template <int D>
constexpr size_t bwd_lds() {
  return MG<D>::at_bytes + 2 * MG<D>::tt_bytes + kGatherLds;
}

// ---------------------------------------------------------------------------
// Forward: Y = relu((A_hat X) W^k)  [+ t = Y w_out^k], with asynchronous global -> LDS
// copies.  (Width 64 runs on the wave-per-tile kernels instead.)
// ---------------------------------------------------------------------------
// A tile moves 16 KB and a memory round trip takes about 2 us, so a workgroup
// that waits for its own loads keeps far too few bytes in flight.  Here the
// rows a tile needs (its own rows, the rows of its first ER entries, its
// entries and its diagonal) are copied straight from HBM into an LDS ring by
// global_load_lds (no registers involved), two tiles ahead of the tile being
// summed and multiplied.
//
// The copies are issued from inline assembly, because the compiler would
// otherwise wait for ALL outstanding copies before any LDS read.  Vector memory
// operations of a wave complete in issue order, so "the copies of tile q have
// landed" is s_waitcnt vmcnt(N) with N = the number of vector memory
// instructions this wave issued after them.  Every N below counts only
// instructions that are certain to have been issued (the copies themselves and
// the unconditional stores); any other load or store issued in between only
// makes the wait stricter, never too weak.  Compiler-generated waits for
// ordinary loads stay correct for the same reason.
__device__ __forceinline__ uint32_t lds_offset(const void* p) {
  return static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
      (__attribute__((address_space(3))) const void*)p));
}

// Each lane copies 16 bytes from its own global address to lds_base + 16 * lane.
__device__ __forceinline__ void dma16(const void* g, uint32_t lds_base) {
  uint32_t keep;  // M0 (the LDS base of the copy) is put back, the compiler may hold a value in it
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
               : "=&s"(keep)
               : "v"(g), "s"(__builtin_amdgcn_readfirstlane(lds_base))
               : "memory");
}
// Each lane copies 4 bytes from its own global address to lds_base + 4 * lane.
__device__ __forceinline__ void dma4(const void* g, uint32_t lds_base) {
  uint32_t keep;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\tglobal_load_lds_dword %1, off\n\ts_mov_b32 m0, %0"
               : "=&s"(keep)
               : "v"(g), "s"(__builtin_amdgcn_readfirstlane(lds_base))
               : "memory");
}

// s_waitcnt vmcnt(n) for a wave-uniform n; n above 24 is clamped (a stricter wait).
__device__ __forceinline__ void wait_vm(int n) {
#define GCO_W(k) case k: asm volatile("s_waitcnt vmcnt(" #k ")" ::: "memory"); break;
  switch (n < 24 ? n : 24) {
    GCO_W(0) GCO_W(1) GCO_W(2) GCO_W(3) GCO_W(4) GCO_W(5) GCO_W(6) GCO_W(7) GCO_W(8)
    GCO_W(9) GCO_W(10) GCO_W(11) GCO_W(12) GCO_W(13) GCO_W(14) GCO_W(15) GCO_W(16)
    GCO_W(17) GCO_W(18) GCO_W(19) GCO_W(20) GCO_W(21) GCO_W(22) GCO_W(23) GCO_W(24)
  }
#undef GCO_W
}

constexpr int kStages = 3;       // LDS ring: the tile being worked on and two in flight
constexpr int kEntBufs = 6;      // entry buffers: tiles q .. q+4 (one spare)
constexpr int kEntStage = 256;   // entries of a tile copied to LDS (tiles with more use HBM)

template <int D>
struct DG {
  static constexpr int ROWB = D * 2;                       // bytes of a feature row
  static constexpr int LPR = D / 8;                        // lanes per row
  static constexpr int EPI = 64 / LPR;                     // rows per copy instruction
  static constexpr int ER = D == 128 ? 40 : (D == 64 ? 72 : 80); // entry rows staged per tile
  static constexpr int NO = R * ROWB / 1024;               // copy instructions for the own rows
  static constexpr int NE = ER / EPI;                      // ... for the entry rows
  static_assert(ER % EPI == 0 && (R * ROWB) % 1024 == 0, "whole copy instructions");
  static constexpr int own_off = 0;
  static constexpr int ent_off = R * ROWB;
  static constexpr int diag_off = (R + ER) * ROWB;
  static constexpr int slot_bytes = diag_off + R * 4;
  static_assert(slot_bytes >= kBlock * 8 * 4, "the slot doubles as the reduction buffer");
  // instructions of one tile's row copies issued by wave w
  __device__ static constexpr int rows_count(int w) {
    return (NO - w + 3) / 4 + (NE - w + 3) / 4 + (w == 0 ? 1 : 0);
  }
  __device__ static constexpr int ents_count(int w) { return w < kEntStage / 128 ? 1 : 0; }
};

template <int D>
constexpr size_t fwd_dma_lds() {
  return static_cast<size_t>(kStages) * DG<D>::slot_bytes + kEntBufs * kEntStage * sizeof(int2) +
         MG<D>::at_bytes + kMaxTilesPerBlock * (R + 1) * sizeof(int) + (R + 4) * sizeof(int) +
         D * sizeof(float);
}

// Copy kEntStage entries, starting at the tile's first entry rounded down to an even
// index (16-byte aligned source), to `buf`: entry e of the tile is buf[e - (e_base & ~1)].
__device__ __forceinline__ void issue_entries(const GraphView& g, int e_base, const int2* buf) {
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  if (wave < kEntStage / 128)   // the entry array is padded, so reading past a tile's end is in bounds
    dma16(g.ent + (e_base & ~1) + wave * 128 + 2 * lane, lds_offset(buf) + wave * 1024);
}

// Copy a tile's own rows, the rows of its first ER entries and its diagonal to `slot`.
template <int D>
__device__ __forceinline__ void issue_rows(const GraphView& g, const bf16_t* X, int row0, const int* rpq,
                                           const int2* ebuf, const unsigned char* slot) {
  using G_ = DG<D>;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const uint32_t base = lds_offset(slot);
  const int last = g.n - 1;
#pragma unroll
  for (int j = wave; j < G_::NO; j += 4) {
    const int r = j * G_::EPI + lane / G_::LPR;
    dma16(X + static_cast<size_t>(min(row0 + r, last)) * D + (lane % G_::LPR) * 8,
          base + G_::own_off + j * 1024);
  }
  const int E = rpq[R] - rpq[0], shift = rpq[0] & 1;
#pragma unroll
  for (int j = wave; j < G_::NE; j += 4) {
    const int el = j * G_::EPI + lane / G_::LPR;
    const int colj = (el < E && el + shift < kEntStage) ? ebuf[el + shift].x : 0;
    dma16(X + static_cast<size_t>(colj) * D + (lane % G_::LPR) * 8, base + G_::ent_off + j * 1024);
  }
  if (wave == 0) dma4(g.diag + min(row0 + lane, last), base + G_::diag_off);
}

template <int D>
__global__ __launch_bounds__(kBlock) void fwd_hidden_dma_kernel(
    GraphView g, const bf16_t* __restrict__ X, const float* __restrict__ W, int w_stride,
    bf16_t* __restrict__ Y, const float* __restrict__ w_out, int wout_stride, float* __restrict__ t,
    const float* __restrict__ heavy_partial) {
  using M = MG<D>;
  using G_ = DG<D>;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* ring = smem;
  int2* entbuf = reinterpret_cast<int2*>(ring + kStages * G_::slot_bytes);
  bf16_t* at = reinterpret_cast<bf16_t*>(entbuf + kEntBufs * kEntStage);
  int* rp = reinterpret_cast<int*>(reinterpret_cast<unsigned char*>(at) + M::at_bytes);
  int* hlist = rp + kMaxTilesPerBlock * (R + 1);
  float* wo = reinterpret_cast<float*>(hlist + R + 4);

  const int k = g.blk_k[blockIdx.x];
  if (k < 0) return;
  const int s = g.blk_s[blockIdx.x], S = g.blk_S[blockIdx.x];
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int tn = wave % M::NT, tm0 = wave / M::NT;
  const int grp = tid / M::LPR, c0 = (tid % M::LPR) * 8;
  const int rbeg = g.part_rows[k], rend = g.part_rows[k + 1];
  const int Q = preload_row_pointers(g, rbeg, rend, s, S, rp);
  const float* Wk = W + static_cast<size_t>(k) * w_stride;
  bf16x8 bfrag[M::KS];
#pragma unroll
  for (int ks = 0; ks < M::KS; ++ks) {
    float v[8];
#pragma unroll
    for (int x = 0; x < 8; ++x) v[x] = Wk[(ks * 16 + 8 * (lane / 32) + x) * D + tn * 32 + lane % 32];
    bfrag[ks] = as_frag(pack8(v));
  }
  if (w_out != nullptr && tid < D) wo[tid] = w_out[static_cast<size_t>(k) * wout_stride + tid];
  const PlainB<D> src{X, g.diag};
  const BfSink<D, false> sink{at, nullptr};
  const int cRW = G_::rows_count(wave), cEN = G_::ents_count(wave);
  constexpr int cST = R * M::LPR / kBlock;  // unconditional 16-byte stores of Y per thread and tile
  __syncthreads();                          // row pointers and wo are in LDS (compiler-visible loads done)

  const auto tile_row0 = [&](int q) { return rbeg + (s + q * S) * R; };
  // prologue: entries of tiles 0..3, rows of tiles 0 and 1
  constexpr int kLead = 4;  // entries are requested this many tiles ahead, rows two tiles ahead
  for (int q = 0; q < kLead && q < Q; ++q) issue_entries(g, rp[q * (R + 1)], entbuf + q * kEntStage);
  for (int q = 0; q < 2 && q < Q; ++q) {
    // entries of tile q have landed: younger are the entry copies of the later tiles and
    // the row copies issued so far
    wait_vm((min(Q, kLead) - 1 - q) * cEN + q * cRW);
    __syncthreads();
    issue_rows<D>(g, X, tile_row0(q), rp + q * (R + 1), entbuf + q * kEntStage, ring + q * G_::slot_bytes);
  }
  for (int q = 0; q < Q; ++q) {
    const int row0 = tile_row0(q);
    const int nrows = min(R, rend - row0);
    const int* rpq = rp + q * (R + 1);
    const unsigned char* slot = ring + (q % kStages) * G_::slot_bytes;
    const int2* ebuf = entbuf + (q % kEntBufs) * kEntStage;
    // Issue order of one iteration: entries of q+4, rows of q+2, ..., stores of q.
    // 1. entries of tile q+4
    if (q + kLead < Q)
      issue_entries(g, rp[(q + kLead) * (R + 1)], entbuf + ((q + kLead) % kEntBufs) * kEntStage);
    const int st_younger = (q >= 1 ? cST : 0) + (q >= 2 ? cST : 0);  // stores of tiles q-1, q-2
    const int en_younger = (q + 3 < Q ? cEN : 0) + (q + 4 < Q ? cEN : 0);
    // 2. rows of tile q+2, once its entries (requested two iterations ago) have landed.
    //    Issued after those entries: rows of q and q+1, stores of q-2 and q-1, entries of q+3, q+4.
    if (q + 2 < Q) {
      wait_vm(2 * cRW + st_younger + en_younger);
      __syncthreads();
      issue_rows<D>(g, X, tile_row0(q + 2), rpq + 2 * (R + 1), entbuf + ((q + 2) % kEntBufs) * kEntStage,
                    ring + ((q + 2) % kStages) * G_::slot_bytes);
    }
    // 3. rows of tile q have landed.  Issued after them: stores of q-2, entries of q+3, rows of q+1,
    //    stores of q-1, entries of q+4, rows of q+2.  (For q = 0 the entries of tile 3 are older.)
    wait_vm((q + 1 < Q ? cRW : 0) + (q + 2 < Q ? cRW : 0) + st_younger +
            (q >= 1 ? en_younger : (q + 4 < Q ? cEN : 0)));
    if (tid == 0) hlist[0] = 0;
    __syncthreads();

    // ---- sum phase: A_hat rows of the tile from the staged rows ----
    const int e_base = rpq[0];
    const int e_al = e_base & ~1;                       // ebuf[0] is entry e_al
    const bool staged = rpq[R] - e_al <= kEntStage;     // all entries of the tile are in ebuf
    const float* dg = reinterpret_cast<const float*>(slot + G_::diag_off);
#pragma unroll
    for (int u = 0; u < M::NCH; ++u) {
      const int r = grp + M::G * u;
      float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      bool direct = true;
      if (r < nrows) {
        const int i = row0 + r;
        const int ea = rpq[r], eb = rpq[r + 1];
        const int deg = eb - ea;
        const uint4 own = *reinterpret_cast<const uint4*>(slot + G_::own_off + r * G_::ROWB + c0 * 2);
        if (deg >= kHeavyMin) {
          src.apply(own, dg[r], acc);
          const int h = find_heavy(g, i);
          for (int ch = g.heavy_chunk_ptr[h]; ch < g.heavy_chunk_ptr[h + 1]; ++ch) {
            const float4* pp = reinterpret_cast<const float4*>(heavy_partial + static_cast<size_t>(ch) * D + c0);
            const float4 p0 = pp[0], p1 = pp[1];
            acc[0] += p0.x; acc[1] += p0.y; acc[2] += p0.z; acc[3] += p0.w;
            acc[4] += p1.x; acc[5] += p1.y; acc[6] += p1.z; acc[7] += p1.w;
          }
        } else if (deg > kLightMax) {
          direct = false;
          if (tid % M::LPR == 0) {
            const int qq = atomicAdd(&hlist[0], 1);
            hlist[1 + qq] = r;
          }
        } else {
          src.apply(own, dg[r], acc);
          int e = ea;
          if (staged) {
            const int e_st = min(eb, e_base + G_::ER);  // entries whose rows are in the slot
            for (; e < e_st; ++e) {
              const int el = e - e_base;
              const uint4 raw = *reinterpret_cast<const uint4*>(slot + G_::ent_off + el * G_::ROWB + c0 * 2);
              src.apply(raw, __int_as_float(ebuf[e - e_al].y), acc);
            }
          }
          for (; e < eb; e += 4) {  // the rest comes from HBM, four rows at a time
            uint4 rw[4];
            float s4[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
              rw[x] = make_uint4(0u, 0u, 0u, 0u);
              s4[x] = 0.f;
              if (e + x < eb) {
                const int2 en = staged ? ebuf[e + x - e_al] : g.ent[e + x];
                rw[x] = *reinterpret_cast<const uint4*>(X + static_cast<size_t>(en.x) * D + c0);
                s4[x] = __int_as_float(en.y);
              }
            }
#pragma unroll
            for (int x = 0; x < 4; ++x) src.apply(rw[x], s4[x], acc);
          }
        }
      }
      if (direct) sink.template put_vec<8>(r, c0, acc);
    }
    __syncthreads();
    {  // rows longer than kLightMax: all lane groups together, entries from HBM
      const int nh = hlist[0];
      float* red = reinterpret_cast<float*>(const_cast<unsigned char*>(slot));  // the slot is spent
      for (int qm = 0; qm < nh; ++qm) {
        const int r = hlist[1 + qm];
        const int i = row0 + r;
        const int ea = rpq[r], eb = rpq[r + 1];
        float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (grp == 0) {
          const uint4 self = *reinterpret_cast<const uint4*>(X + static_cast<size_t>(i) * D + c0);
          src.apply(self, g.diag[i], a8);
        }
        for (int e = ea + grp; e < eb; e += 4 * M::G) {
          uint4 rw[4];
          float s4[4];
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            const int ee = e + x * M::G;
            rw[x] = make_uint4(0u, 0u, 0u, 0u);
            s4[x] = 0.f;
            if (ee < eb) {
              const int2 en = g.ent[ee];
              rw[x] = *reinterpret_cast<const uint4*>(X + static_cast<size_t>(en.x) * D + c0);
              s4[x] = __int_as_float(en.y);
            }
          }
#pragma unroll
          for (int x = 0; x < 4; ++x) src.apply(rw[x], s4[x], a8);
        }
#pragma unroll
        for (int x = 0; x < 8; ++x) red[grp * D + c0 + x] = a8[x];
        __syncthreads();
        if (tid < D) {
          float sum = 0.f;
          for (int gq = 0; gq < M::G; ++gq) sum += red[gq * D + tid];
          sink.put_one(r, tid, sum);
        }
        __syncthreads();
      }
    }

    // ---- dense product, ReLU, store ----
    floatx16 acc[M::NTM];
    tile_product<D>(at, bfrag, tm0, acc);
    __syncthreads();
#pragma unroll
    for (int qq = 0; qq < M::NTM; ++qq) {
      const int tm = tm0 + qq * M::WPC;
      if (tm < M::MT) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = tm * 32 + (r / 4) * 8 + (lane / 32) * 4 + r % 4;
          at[i * M::PA + tn * 32 + lane % 32] = f32_to_bf16(fmaxf(acc[qq][r], 0.f));
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < cST; ++u) {  // unconditional: rows past the tile are clamped, not skipped
      const int idx = tid + kBlock * u;
      const int r = idx / M::LPR;
      const int rr = min(r, nrows - 1);  // duplicates rewrite the last row with its own values
      *reinterpret_cast<uint4*>(Y + static_cast<size_t>(row0 + rr) * D + c0) =
          *reinterpret_cast<const uint4*>(at + rr * M::PA + c0);
    }
    if (w_out != nullptr) {
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
template <int D, bool LAST>
__device__ __host__ __forceinline__ typename std::conditional<LAST, LastB<D>, PlainB<D>>::type make_src(
    const BwdArgs& a, const GraphView& g) {
  if constexpr (LAST) {
    return LastB<D>{static_cast<const bf16_t*>(a.Hcur), g.diag, a.g_t, a.w_out, a.wout_stride, {}};
  } else {
    return PlainB<D>{static_cast<const bf16_t*>(a.GZ_in), g.diag};
  }
}

template <int D, bool LAST, bool TO_EMBED>
__global__ __launch_bounds__(kBlock) void bwd_hidden_bf16_kernel(GraphView g, BwdArgs a) {
  using M = MG<D>;
  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* at = reinterpret_cast<bf16_t*>(smem);                              // G_T [row][feature]
  bf16_t* gtt = reinterpret_cast<bf16_t*>(smem + M::at_bytes);               // G_T [feature][row]
  bf16_t* hpt = reinterpret_cast<bf16_t*>(smem + M::at_bytes + M::tt_bytes); // Hprev [feature][row]
  float* red = reinterpret_cast<float*>(smem + M::at_bytes + 2 * M::tt_bytes);
  int2* ents = reinterpret_cast<int2*>(red + kBlock * 8);
  int* rp = reinterpret_cast<int*>(ents + kEntCap);
  int* hlist = rp + kMaxTilesPerBlock * (R + 1);
  float* stage = reinterpret_cast<float*>(smem);  // fp32 [R][PO], over at + gtt, after the products

  const int k = g.blk_k[blockIdx.x];
  if (k < 0) return;
  const AdamStep ad = a.adam.for_part(k);
  const int s = g.blk_s[blockIdx.x], S = g.blk_S[blockIdx.x];
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int tn = wave % M::NT, tm0 = wave / M::NT;
  const int rbeg = g.part_rows[k], rend = g.part_rows[k + 1];
  const int Q = preload_row_pointers(g, rbeg, rend, s, S, rp);
  const bf16_t* Hprev = static_cast<const bf16_t*>(a.Hprev);
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
  const int c0 = (tid % M::LPR) * 8;  // this thread's feature slice in row-chunk loops
  using Src = typename std::conditional<LAST, LastB<D>, PlainB<D>>::type;
  Src src = make_src<D, LAST>(a, g);
  src.set_part(k, c0);
  const BfSink<D, true> sink{at, gtt};

  floatx16 gw[M::NGW];
#pragma unroll
  for (int q = 0; q < M::NGW; ++q)
#pragma unroll
    for (int r = 0; r < 16; ++r) gw[q][r] = 0.f;
  float gwo[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  __syncthreads();  // row pointers are in LDS
  TileRegs<D> next;
  uint4 hp_next[M::NCH];
  if (Q > 0) {
    const int nr0 = min(R, rend - (rbeg + s * R));
    prefetch_tile<D>(g, src, rbeg + s * R, nr0, rp, next);
    prefetch_rows<D>(Hprev, rbeg + s * R, nr0, hp_next);
  }
  for (int qt = 0; qt < Q; ++qt) {
    const int row0 = rbeg + (s + qt * S) * R;
    const int nrows = min(R, rend - row0);
    const int* rpq = rp + qt * (R + 1);
    uint4 own[M::NCH], hp[M::NCH];
#pragma unroll
    for (int u = 0; u < M::NCH; ++u) {
      own[u] = next.own[u];
      hp[u] = hp_next[u];
    }
    const bool in_lds = next.in_lds;
    commit_entries<D>(next, ents);
    if (tid == 0) hlist[0] = 0;
    __syncthreads();
    if (qt + 1 < Q) {
      const int row1 = row0 + S * R;
      prefetch_tile<D>(g, src, row1, min(R, rend - row1), rpq + (R + 1), next);
      prefetch_rows<D>(Hprev, row1, min(R, rend - row1), hp_next);
    }
    gather_tile<D>(g, src, sink, row0, nrows, rpq, ents, in_lds, own, red, hlist, a.heavy_partial);
    // Hprev tile (prefetched), transposed into LDS; zero beyond the tile's rows
#pragma unroll
    for (int u = 0; u < M::NCH; ++u) {
      const int r = tid / M::LPR + M::G * u;
      const uint32_t w[4] = {hp[u].x, hp[u].y, hp[u].z, hp[u].w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        hpt[(c0 + 2 * q) * M::PT + r] = static_cast<bf16_t>(w[q] & 0xffffu);
        hpt[(c0 + 2 * q + 1) * M::PT + r] = static_cast<bf16_t>(w[q] >> 16);
      }
      if (LAST && r < nrows) {  // gradient of w_out: sum_r Hcur[r, c] * g_t[r]
        float h[8];
        unpack8(own[u], h);
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
              mo[x] = ad.b1 * mv[x] + (1.f - ad.b1) * gv[x];
              vo[x] = ad.b2 * vv[x] + (1.f - ad.b2) * gv[x] * gv[x];
              const float upd = (mo[x] * ad.inv_bc1) / (sqrtf(vo[x]) * ad.inv_sqrt_bc2 + ad.eps);
              eo[x] = ev[x] - ad.lr * upd;
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
    const PlainB<D> src{static_cast<const bf16_t*>(X), g.diag};
    heavy_wide_b_kernel<D, PlainB<D>><<<g.num_chunks, kBlock, 0, ln.st>>>(g, src, heavy_partial);
    ln.end(KK_HEAVY);
  }
  if (D == 64 || D == 128) {  // wave-per-tile kernel
    launch_fwd_hidden_wave(ln, D, g, X, W, w_stride, Y, w_out, wout_stride, t, heavy_partial);
    return;
  }
  allow_lds(fwd_hidden_dma_kernel<D>, fwd_dma_lds<D>());
  ln.begin(KK_FWD_HIDDEN);
  fwd_hidden_dma_kernel<D><<<g.num_blocks, kBlock, fwd_dma_lds<D>(), ln.st>>>(
      g, static_cast<const bf16_t*>(X), W, w_stride, static_cast<bf16_t*>(Y), w_out, wout_stride, t,
      heavy_partial);
  ln.end(KK_FWD_HIDDEN);
}

template <int D>
void bwd_t(const Launch& ln, bool last, bool to_embed, const GraphView& gt, const BwdArgs& a) {
  if (D == 64 || D == 128) {  // wave-per-tile kernels: G_Z of the last layer is formed first
    BwdArgs b = a;
    if (last) {
      launch_form_gz_last(ln, D, gt, a);
      b.GZ_in = a.GZ_last;
    }
    if (gt.num_chunks > 0) {
      ln.begin(KK_HEAVY);
      const PlainB<D> src{static_cast<const bf16_t*>(b.GZ_in), gt.diag};
      heavy_wide_b_kernel<D, PlainB<D>><<<gt.num_chunks, kBlock, 0, ln.st>>>(gt, src, a.heavy_partial);
      ln.end(KK_HEAVY);
    }
    launch_bwd_hidden_wave(ln, D, to_embed, gt, b);
    return;
  }
  if (gt.num_chunks > 0) {
    ln.begin(KK_HEAVY);
    if (last) {
      const LastB<D> src{static_cast<const bf16_t*>(a.Hcur), gt.diag, a.g_t, a.w_out, a.wout_stride, {}};
      heavy_wide_b_kernel<D, LastB<D>><<<gt.num_chunks, kBlock, 0, ln.st>>>(gt, src, a.heavy_partial);
    } else {
      const PlainB<D> src{static_cast<const bf16_t*>(a.GZ_in), gt.diag};
      heavy_wide_b_kernel<D, PlainB<D>><<<gt.num_chunks, kBlock, 0, ln.st>>>(gt, src, a.heavy_partial);
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
