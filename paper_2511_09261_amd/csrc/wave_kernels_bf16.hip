// Wave-per-tile bf16 layer kernels (widths 64 and 128).
//
// Every 64-lane wavefront owns a contiguous run of 32-row tiles of one subgraph
// and works through it alone: there is no workgroup barrier after the prologue,
// so the wavefronts of a compute unit overlap each other's memory round trips
// freely.  The four wavefronts of a workgroup only share the LDS copy of their
// subgraph's weight matrix.
//
// The aggregation A_hat X is driven by the light stream: the entries of all rows
// that are not pre-reduced, each row's list led by its diagonal entry {i, A_hat_ii},
// row after row; an entry's value is kept as two bf16 numbers hi + lo (relative
// error 2^-17).  A wavefront's tiles own a contiguous range of that stream, which
// it consumes in steps of SE entries ("slots"), whatever the row lengths:
//   * lane group g (the lanes that share one 16-byte-per-lane feature row) fetches
//     the source rows of slots 8g .. 8g+7 together with the entries of the next
//     step -- one full wait per step, all loads of the step in flight together;
//   * the rows go to a wave-private LDS buffer transposed ([feature][slot]), from
//     which every lane reads matrix-core fragments: 8 consecutive slots of one
//     feature;
//   * the sum over each row's entries is a product on the matrix cores,
//         AGG^T[feature, row] += sum_slot X[slot, feature] * S[slot, row],
//     with S[slot, row] = the entry's value if the slot belongs to the row, else 0
//     (once with the hi parts and once with the lo parts): its cost does not depend
//     on how the entries are spread over the rows;
//   * when a step reaches the end of a tile's entries the tile is complete:
//     pre-reduced rows add their chunk partials and the caller's dense part runs
//     on the fp32 accumulators; the step's remaining slots belong to the next tile.
// Row pointers of the next two tiles are requested ahead.  The LDS traffic of one
// wavefront needs no barrier: its LDS operations execute in program order.
//
// v_mfma_f32_32x32x16_bf16, lane l = (n = l % 32, h = l / 32):
//   A operand: row n of the left matrix, contraction indices 8h .. 8h+7
//   B operand: column n of the right matrix, contraction indices 8h .. 8h+7
//   C/D register r: row 8 (r/4) + 4h + r%4, column n
// AGG^T therefore leaves the first product with lane (n, h) holding, for row n of the
// tile, features 32 tn + 8i + 4h + {0..3} (i = 0..3) -- exactly a B operand of the
// second product Z^T = W^T AGG^T if contraction index 8h + e of its step (tn, p)
// stands for feature 32 tn + 16 p + 8 (e/4) + 4h + e%4; the LDS copy of W^k is laid
// out in that order, so the aggregate never leaves the registers.
#include "bf16_common.h"
#include "device_utils.h"
#include "gco_internal.h"
#include "heavy_chunk.h"

namespace gco {
namespace {

constexpr int RW = kWaveRows;
static_assert(RW == 32, "one 32-row matrix-core tile per wavefront tile");

template <int D>
struct WG {
  static constexpr int LPR = D / 8;      // lanes per feature row (16 bytes each)
  static constexpr int NG = 64 / LPR;    // lane groups per wavefront
  static constexpr int SE = 8 * NG;      // slots (entries) per step
  static constexpr int KS1 = SE / 16;    // contraction steps over the slots
  static constexpr int NT = D / 32;      // 32-wide feature tiles
  static constexpr int KS2 = D / 16;     // contraction steps over the features
  static constexpr int NO = RW / NG;     // output rows per lane group
  static constexpr int XP = SE * 2 + 16; // bytes per feature in the transposed row buffer
  static constexpr int PA = D + 8;       // pitch of the bf16 output tile
  static constexpr int GP = RW * 2 + 16; // bytes per feature of a transposed 32-row bf16 tile
  static constexpr int PF = D + 4;       // pitch (floats) of an fp32 32-row tile
  // Width 64: the weight-gradient accumulators (D*D/64 registers per lane) stay in the
  // backward kernel.  Width 128: they do not fit, the backward kernel stores G_T and a
  // kernel of its own forms the weight gradient.
  static constexpr bool GW_INLINE = D <= 64;
  // one wave-private LDS region serves, in turn, as the transposed row buffer of a step,
  // as the two transposed tiles of the weight-gradient product, and as the output tile
  static constexpr size_t xf_bytes = static_cast<size_t>(D) * XP;  // forward: row buffer / output tile
  static constexpr size_t two_tiles = static_cast<size_t>(D) * (XP > 2 * GP ? XP : 2 * GP);
  static constexpr size_t region_bytes =                           // backward
      !GW_INLINE ? xf_bytes
                 : (two_tiles > static_cast<size_t>(RW) * PF * 4 ? two_tiles : static_cast<size_t>(RW) * PF * 4);
  // the fp32 gradient rows of the embedding pass through the region whole, or in two halves
  static constexpr int SP = static_cast<size_t>(RW) * PF * 4 <= region_bytes ? 1 : 2;
  static constexpr int RS = RW / SP;
  static_assert(static_cast<size_t>(RS) * PF * 4 <= region_bytes, "staging of the embedding gradient");
  static constexpr size_t wts_bytes = static_cast<size_t>(SE) * 4;  // hi halves, then lo halves
  static constexpr size_t ot_bytes = static_cast<size_t>(RW) * PA * 2;
  // the output tile reuses the row buffer: the step's fragments are in registers by then
  static constexpr size_t wave_bytes = xf_bytes + wts_bytes;
  // width 128: the backward kernels keep the next step's entries in LDS
  static constexpr bool BWD_LDS_ENTRIES = D == 128;
  static constexpr size_t ent_bytes = static_cast<size_t>(SE) * 8;
  static constexpr size_t bwd_wave_bytes = region_bytes + wts_bytes + (BWD_LDS_ENTRIES ? ent_bytes : 0);
  static_assert(ot_bytes <= xf_bytes && ot_bytes <= region_bytes, "the output tile overlays the row buffer");
  static constexpr size_t w_bytes = static_cast<size_t>(D) * D * 2;
  static_assert(SE <= 64, "slot masks are 64 bits wide");
  static_assert(wave_bytes % 16 == 0 && w_bytes % 16 == 0 && XP % 16 == 0, "alignment");
  static_assert(2 * SE <= kEntPad, "the stream is read up to two steps past a wavefront's range");
};

// Feature that contraction index (h, e) of step ks2 of the second product stands for.
__host__ __device__ constexpr int feature_of(int ks2, int h, int e) {
  return 32 * (ks2 / 2) + 16 * (ks2 % 2) + 8 * (e / 4) + 4 * h + e % 4;
}

// Feature held in register r of accumulator tile tn by a lane of half h.
__host__ __device__ constexpr int acc_feature(int tn, int h, int r) { return 32 * tn + 8 * (r / 4) + 4 * h + r % 4; }

// W^k (fp32 [D][D] in HBM) -> LDS as A operands of Z^T = W^T AGG^T:
// wfr[((tj * KS2 + ks2) * 64 + lane) * 8 + e] = W[feature_of(ks2, h, e)][32 tj + n].
template <int D>
__device__ __forceinline__ void load_weight_fragments(const float* __restrict__ Wk, bf16_t* wfr) {
  constexpr int kPer = D * D / 4 / kBlock;  // float4 loads per thread
  static_assert(D * D % (4 * kBlock) == 0, "whole float4 loads");
  float4 v[kPer];
#pragma unroll
  for (int q = 0; q < kPer; ++q) v[q] = reinterpret_cast<const float4*>(Wk)[threadIdx.x + q * kBlock];
#pragma unroll
  for (int q = 0; q < kPer; ++q) {
    const int idx = (threadIdx.x + q * kBlock) * 4;
    const int f = idx / D, j0 = idx % D;  // W[f][j0 .. j0+3]
    // inverse of feature_of: f = 32 tn + 16 p + 8 (e/4) + 4 h + e%4
    const int ks2 = f / 16, h = (f / 4) % 2, e = ((f / 8) % 2) * 4 + f % 4;
    const float w[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int j = j0 + x;
      wfr[(((j / 32) * WG<D>::KS2 + ks2) * 64 + h * 32 + j % 32) * 8 + e] = f32_to_bf16(w[x]);
    }
  }
}

// W^k -> LDS as A operands of G_H^T = W G_T^T:
// wfr[((ta * KS2 + ks2) * 64 + lane) * 8 + e] = W[32 ta + n][feature_of(ks2, h, e)].
template <int D>
__device__ __forceinline__ void load_weight_fragments_t(const float* __restrict__ Wk, bf16_t* wfr) {
  constexpr int kPer = D * D / 4 / kBlock;
  float4 v[kPer];
#pragma unroll
  for (int q = 0; q < kPer; ++q) v[q] = reinterpret_cast<const float4*>(Wk)[threadIdx.x + q * kBlock];
#pragma unroll
  for (int q = 0; q < kPer; ++q) {
    const int idx = (threadIdx.x + q * kBlock) * 4;
    const int a = idx / D, b0 = idx % D;  // W[a][b0 .. b0+3]: one run e%4 = 0..3 of feature_of
    const int ks2 = b0 / 16, h = (b0 / 4) % 2, e0 = ((b0 / 8) % 2) * 4;
    uint2 pk;
    pk.x = f32x2_to_bf16x2(v[q].x, v[q].y);
    pk.y = f32x2_to_bf16x2(v[q].z, v[q].w);
    *reinterpret_cast<uint2*>(wfr + (((a / 32) * WG<D>::KS2 + ks2) * 64 + h * 32 + a % 32) * 8 + e0) = pk;
  }
}

// pair_mask[b] for an 8-bit pattern b: four words whose 16-bit halves are all ones where
// the corresponding bit of b is set (bit 2d -> lower half of word d).
__device__ __forceinline__ void fill_pair_masks(uint4* pair_mask) {
  for (int b = threadIdx.x; b < 256; b += kBlock) {
    uint32_t d[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
      d[q] = ((b >> (2 * q)) & 1 ? 0xffffu : 0u) | ((b >> (2 * q + 1)) & 1 ? 0xffff0000u : 0u);
    pair_mask[b] = make_uint4(d[0], d[1], d[2], d[3]);
  }
}

// Lower (upper) halves of two words, x first.
__device__ __forceinline__ uint32_t lower_halves(uint32_t x, uint32_t y) {
  return __builtin_amdgcn_perm(y, x, 0x05040100u);
}
__device__ __forceinline__ uint32_t upper_halves(uint32_t x, uint32_t y) {
  return __builtin_amdgcn_perm(y, x, 0x07060302u);
}

// ---- copies from global memory straight into LDS (no register receives the data) ----
__device__ __forceinline__ uint32_t lds_offset(const void* p) {
  return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const void*)p));
}
// Each lane copies 16 bytes from its own global address to lds_base + 16 * lane.  The copy is
// one of the wavefront's vector memory operations (they complete in the order issued), but
// the compiler does not know what it writes: whoever reads the LDS bytes waits by hand.
__device__ __forceinline__ void load_to_lds_16(const void* gp, uint32_t lds_base) {
  uint32_t keep;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
               : "=&s"(keep)
               : "v"(gp), "s"(__builtin_amdgcn_readfirstlane(lds_base))
               : "memory");
}
// The same with 4 bytes per lane, to lds_base + 4 * lane.
__device__ __forceinline__ void load_to_lds_4(const void* gp, uint32_t lds_base) {
  uint32_t keep;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\tglobal_load_lds_dword %1, off\n\ts_mov_b32 m0, %0"
               : "=&s"(keep)
               : "v"(gp), "s"(__builtin_amdgcn_readfirstlane(lds_base))
               : "memory");
}

template <bool FIRST, typename A, typename B>
__device__ __forceinline__ auto& select_array(A& a, B& b) {
  if constexpr (FIRST) return a;
  else return b;
}

// Calls on_tile(row0, nrows, agg) for every tile of the wavefront's run, in order.  agg[tn][r] at lane (n, h) is element (row0 + n, acc_feature(tn, h, r)) of
// A_hat X in fp32 (zero for rows past nrows).  `went` is the light stream of the matrix
// that is applied (A_hat or its transpose); xf (xf_bytes) and wts (wts_bytes) are this
// wavefront's LDS; pair_mask is the workgroup's table from fill_pair_masks.  on_tile may
// overwrite xf.
// EARLY_ROWS: the source rows of a step are requested during the step before it, as soon as
// that step's rows are parked in LDS (their registers are free again), together with the
// entries of the step after; the products and tile epilogues of a step then run beside the
// next step's round trip.  The rows in flight occupy 32 registers through the epilogue and
// the entries another 16: for the kernel that has them to spare (forward, width 128).
// LDS_ENTRIES (not with EARLY_ROWS): the entries of the next step are copied straight into
// ent_lds (8 * SE bytes of this wavefront's LDS) instead of into 16 registers that stay live
// through the whole step, and are read from there when the step ends.  The copy is issued
// before the step's row requests, so it has landed when the rows have (vector memory
// operations complete in order); the kernels at the register limit use it.
template <int D, bool EARLY_ROWS, bool LDS_ENTRIES, typename OnTile>
__device__ __forceinline__ void stream_tiles(const GraphView& g, const int2* __restrict__ went,
                                             const bf16_t* __restrict__ X, const WaveRun& run,
                                             unsigned char* xf, uint32_t* wts, const uint4* pair_mask,
                                             const float* __restrict__ heavy_partial, unsigned char* ent_lds,
                                             OnTile&& on_tile) {
  using G_ = WG<D>;
  static_assert(!(EARLY_ROWS && LDS_ENTRIES), "one way of prefetching entries at a time");
  const int lane = threadIdx.x % 64;
  const int n = lane % 32, h = lane / 32;
  const int grp = lane / G_::LPR, sub = lane % G_::LPR;

  const int tile0 = run.tile0, tile1 = run.tile1;
  const int rbeg = run.rbeg, rend = run.rend;
  const int E0 = run.e0, E1 = run.e1;
  const int tglob = run.tglob;
  // Lane-held facts of tile tau: lanes 0..32 the stream offsets of its rows (clamped to
  // the tile's end), lanes 33 and 34 its range in the list of pre-reduced rows.
  auto tile_facts = [&](int tau) -> int {
    if (tau >= tile1) return 0;
    const int r0 = rbeg + tau * RW, nr = min(RW, rend - r0);
    const int* p = g.wrowptr + r0 + min(lane, nr);
    if (lane == RW + 1 || lane == RW + 2) p = g.wtile_hptr + tglob + tau + (lane - RW - 1);
    return *p;
  };
  int factsA = tile_facts(tile0), factsB = tile_facts(tile0 + 1), factsC = tile_facts(tile0 + 2);
  int tau = tile0;
  int row0 = rbeg + tau * RW, nrows = min(RW, rend - row0);
  int te0 = __builtin_amdgcn_readlane(factsA, 0), te1 = __builtin_amdgcn_readlane(factsA, nrows);
  int ra = __shfl(factsA, n, 64), rb = __shfl(factsA, n + 1, 64);  // stream range of row n of the tile
  floatx16 agg[G_::NT];
#pragma unroll
  for (int tn = 0; tn < G_::NT; ++tn)
#pragma unroll
    for (int r = 0; r < 16; ++r) agg[tn][r] = 0.f;

  int2 cur[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) cur[j] = went[E0 + grp * 8 + j];
  // The first entries are taken here, before the loop.  Inside the loop the entries of a
  // step arrive together with the rows of the step before; if the compiler had to allow
  // for these first loads still being on their way at the top of the loop, it would put a
  // wait there that, vector memory operations completing in order, also waits for the
  // stores of the tile epilogue just before -- ahead of the row requests instead of
  // beside them.
  asm volatile("" ::"v"(cur[0].x), "v"(cur[1].x), "v"(cur[2].x), "v"(cur[3].x), "v"(cur[4].x), "v"(cur[5].x),
               "v"(cur[6].x), "v"(cur[7].x), "v"(cur[0].y), "v"(cur[1].y), "v"(cur[2].y), "v"(cur[3].y),
               "v"(cur[4].y), "v"(cur[5].y), "v"(cur[6].y), "v"(cur[7].y));

  // rows of the step that starts at entry b: 8 slots per lane group, 16 bytes per lane
  auto request_rows = [&](uint4 (&rows)[8], const int2 (&ent)[8], int b) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      rows[j] = make_uint4(0u, 0u, 0u, 0u);
      if (b + grp * 8 + j < E1)
        rows[j] = *reinterpret_cast<const uint4*>(X + static_cast<size_t>(ent[j].x) * D + sub * 8);
    }
  };
  static_assert(kEntPad >= 3 * G_::SE, "entries are read up to two steps past the end of the stream");
  // what EARLY_ROWS carries from one step to the next (unused otherwise)
  int2 nxt_carried[EARLY_ROWS ? 8 : 1];
  uint4 raw_carried[EARLY_ROWS ? 8 : 1];
  if constexpr (EARLY_ROWS) {
#pragma unroll
    for (int j = 0; j < 8; ++j) nxt_carried[j] = went[E0 + G_::SE + grp * 8 + j];
    request_rows(raw_carried, cur, E0);
  }
  for (int b0 = E0; b0 < E1; b0 += G_::SE) {
    int2 nxt_here[EARLY_ROWS || LDS_ENTRIES ? 1 : 8];
    uint4 raw_here[EARLY_ROWS ? 1 : 8];
    if constexpr (LDS_ENTRIES) {
      // the previous contents of ent_lds have been read (the reads were issued a step ago)
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      const uint32_t ent_base = lds_offset(ent_lds);
#pragma unroll
      for (int i = 0; i < G_::SE * 2 / 64; ++i)
        load_to_lds_4(reinterpret_cast<const uint32_t*>(went + b0 + G_::SE) + i * 64 + lane, ent_base + i * 256);
      request_rows(raw_here, cur, b0);
    } else if constexpr (!EARLY_ROWS) {
      // the next step's entries and this step's source rows: one round trip
#pragma unroll
      for (int j = 0; j < 8; ++j) nxt_here[j] = went[b0 + G_::SE + grp * 8 + j];
      request_rows(raw_here, cur, b0);
    }
    auto& nxt = select_array<EARLY_ROWS>(nxt_carried, nxt_here);
    auto& raw = select_array<EARLY_ROWS>(raw_carried, raw_here);
    // transpose in the lane (8 slots x 8 features) and park as [feature][slot]
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      uint32_t d[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t x = (&raw[2 * q].x)[i / 2], y = (&raw[2 * q + 1].x)[i / 2];
        d[q] = (i % 2 == 0) ? lower_halves(x, y) : upper_halves(x, y);
      }
      // the 16-byte groups of a feature are rotated by feature / 8, so that the lanes of
      // one store (features 8 apart) fall into different LDS banks
      *reinterpret_cast<uint4*>(xf + (sub * 8 + i) * G_::XP + ((grp + sub) % G_::NG) * 16) =
          make_uint4(d[0], d[1], d[2], d[3]);
    }
    if (sub == 0) {  // values of slots 8 grp .. 8 grp + 7: the hi halves, the lo halves
      const uint32_t y[8] = {static_cast<uint32_t>(cur[0].y), static_cast<uint32_t>(cur[1].y),
                             static_cast<uint32_t>(cur[2].y), static_cast<uint32_t>(cur[3].y),
                             static_cast<uint32_t>(cur[4].y), static_cast<uint32_t>(cur[5].y),
                             static_cast<uint32_t>(cur[6].y), static_cast<uint32_t>(cur[7].y)};
      *reinterpret_cast<uint4*>(wts + grp * 4) = make_uint4(upper_halves(y[0], y[1]), upper_halves(y[2], y[3]),
                                                            upper_halves(y[4], y[5]), upper_halves(y[6], y[7]));
      *reinterpret_cast<uint4*>(wts + G_::SE / 2 + grp * 4) =
          make_uint4(lower_halves(y[0], y[1]), lower_halves(y[2], y[3]), lower_halves(y[4], y[5]),
                     lower_halves(y[6], y[7]));
    }
    int2 nx2[8];
    if constexpr (EARLY_ROWS) {
      request_rows(raw, nxt, b0 + G_::SE);
#pragma unroll
      for (int j = 0; j < 8; ++j) nx2[j] = went[b0 + 2 * G_::SE + grp * 8 + j];
    }
    wave_lds_handoff();
    // fragments of the step: slots 16 ks + 8h .. + 7 of feature 32 tn + n, and their values
    bf16x8 xa[G_::NT][G_::KS1];
    {
      // the fragment addresses are worked out again in every step (a few integer operations):
      // held in registers across the whole step they are the first to be spilled
      int nf = n;
      asm volatile("" : "+v"(nf));
#pragma unroll
      for (int tn = 0; tn < G_::NT; ++tn)
#pragma unroll
        for (int ks = 0; ks < G_::KS1; ++ks)
          xa[tn][ks] = as_frag(*reinterpret_cast<const uint4*>(
              xf + (tn * 32 + nf) * G_::XP + ((2 * ks + h + (tn * 32 + nf) / 8) % G_::NG) * 16));
    }
    const int b1 = min(b0 + G_::SE, E1);
    while (true) {
      // slots of the step that belong to row n of the current tile, as a bit mask
      const int mlo = min(max(ra - b0, 0), G_::SE), mhi = min(max(rb - b0, 0), G_::SE);
      unsigned long long m64 = 0ull;
      if (mlo < mhi) m64 = (mhi >= 64 ? ~0ull : ((1ull << mhi) - 1ull)) & ~((1ull << mlo) - 1ull);
      m64 >>= 8 * h;
      const int tlo = max(te0, b0) - b0, thi = min(te1, b1) - b0;  // the tile's slots in this step
#pragma unroll
      for (int ks = 0; ks < G_::KS1; ++ks) {
        if (16 * ks < thi && 16 * ks + 16 > tlo) {
          uint4 shi = *reinterpret_cast<const uint4*>(wts + (2 * ks + h) * 4);
          uint4 slo = *reinterpret_cast<const uint4*>(wts + G_::SE / 2 + (2 * ks + h) * 4);
          const uint32_t half = static_cast<uint32_t>(m64 >> (ks >= 2 ? 32 : 0));
          const uint4 pm = pair_mask[(half >> ((16 * ks) % 32)) & 0xffu];
          shi.x &= pm.x; shi.y &= pm.y; shi.z &= pm.z; shi.w &= pm.w;
          slo.x &= pm.x; slo.y &= pm.y; slo.z &= pm.z; slo.w &= pm.w;
#pragma unroll
          for (int tn = 0; tn < G_::NT; ++tn) {
            agg[tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[tn][ks], as_frag(shi), agg[tn], 0, 0, 0);
            agg[tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[tn][ks], as_frag(slo), agg[tn], 0, 0, 0);
          }
        }
      }
      if (te1 > b1) break;  // the tile goes on in the next step
      // the tile is complete: pre-reduced rows take their chunk partials
      const int h0 = __builtin_amdgcn_readlane(factsA, RW + 1), h1 = __builtin_amdgcn_readlane(factsA, RW + 2);
      for (int hh = h0; hh < h1; ++hh) {
        // the whole wavefront sums the row's chunk partials: lane (cg, fq) = (lane / LQ,
        // lane % LQ) adds chunks cg, cg + CG, ... for features 4 fq .. 4 fq + 3, four loads
        // in flight; the CG groups are then added in order
        constexpr int LQ = D / 4, CG = 64 / LQ;
        const int c0h = g.heavy_chunk_ptr[hh], c1h = g.heavy_chunk_ptr[hh + 1];
        float4 tot = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int ch = c0h + lane / LQ; ch < c1h; ch += 4 * CG) {
          float4 pv[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            pv[c] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (ch + c * CG < c1h)
              pv[c] = *reinterpret_cast<const float4*>(heavy_partial + static_cast<size_t>(ch + c * CG) * D +
                                                       (lane % LQ) * 4);
          }
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            tot.x += pv[c].x; tot.y += pv[c].y; tot.z += pv[c].z; tot.w += pv[c].w;
          }
        }
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int cg = 0; cg < CG; ++cg) {
          sum.x += __shfl(tot.x, cg * LQ + lane % LQ, 64);
          sum.y += __shfl(tot.y, cg * LQ + lane % LQ, 64);
          sum.z += __shfl(tot.z, cg * LQ + lane % LQ, 64);
          sum.w += __shfl(tot.w, cg * LQ + lane % LQ, 64);
        }
        // hand the totals to the two lanes that hold the row
        const bool mine = g.heavy_rows[hh] - row0 == n;
#pragma unroll
        for (int tn = 0; tn < G_::NT; ++tn)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int src = acc_feature(tn, h, 4 * i) / 4;
            const float x0 = __shfl(sum.x, src, 64), x1 = __shfl(sum.y, src, 64);
            const float x2 = __shfl(sum.z, src, 64), x3 = __shfl(sum.w, src, 64);
            if (mine) {
              agg[tn][4 * i] += x0; agg[tn][4 * i + 1] += x1;
              agg[tn][4 * i + 2] += x2; agg[tn][4 * i + 3] += x3;
            }
          }
      }
      on_tile(row0, nrows, agg);
      wave_lds_handoff();
#pragma unroll
      for (int tn = 0; tn < G_::NT; ++tn)
#pragma unroll
        for (int r = 0; r < 16; ++r) agg[tn][r] = 0.f;
      // next tile
      ++tau;
      if (tau >= tile1) break;
      factsA = factsB;
      factsB = factsC;
      factsC = tile_facts(tau + 2);
      row0 = rbeg + tau * RW;
      nrows = min(RW, rend - row0);
      te0 = te1;
      te1 = __builtin_amdgcn_readlane(factsA, nrows);
      ra = __shfl(factsA, n, 64);
      rb = __shfl(factsA, n + 1, 64);
    }
    if constexpr (LDS_ENTRIES) {
      // after this step's rows, which were requested after the copy, have been used
      asm volatile("" ::: "memory");
#pragma unroll
      for (int j = 0; j < 8; ++j) cur[j] = reinterpret_cast<const int2*>(ent_lds)[grp * 8 + j];
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) cur[j] = nxt[j];
    }
    if constexpr (EARLY_ROWS) {
#pragma unroll
      for (int j = 0; j < 8; ++j) nxt[j] = nx2[j];
    }
    wave_lds_handoff();
  }
}

// 16-byte accesses marked non-temporal: loads of data that is streamed once (optimizer
// state, own rows read once), so that they do not displace the gathered rows from the
// caches, and the stores of whole output rows, which complete sooner that way (a
// wavefront's next wait for loads also waits for its earlier stores).
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_streamed(const float* p) {
  const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_streamed(const bf16_t* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_streamed(float* p, float a, float b, float c, float d) {
  const f32x4_t v = {a, b, c, d};
  __builtin_nontemporal_store(v, reinterpret_cast<f32x4_t*>(p));
}

__device__ __forceinline__ void store_streamed(bf16_t* p, const uint4& q) {
  const u32x4_t v = {q.x, q.y, q.z, q.w};
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(p));
}

template <int D>
constexpr size_t fwd_wave_lds() {
  return WG<D>::w_bytes + D * sizeof(float) + 256 * sizeof(uint4) + 4 * WG<D>::wave_bytes;
}

// ---------------------------------------------------------------------------
// Forward: Y = relu((A_hat X) W^k)  [+ t = Y w_out^k]
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kBlock, D == 64 ? 3 : 2) void fwd_wave_kernel(
    GraphView g, const bf16_t* __restrict__ X, const float* __restrict__ W, int w_stride,
    bf16_t* __restrict__ Y, const float* __restrict__ w_out, int wout_stride, float* __restrict__ t,
    const float* __restrict__ heavy_partial) {
  using G_ = WG<D>;
  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* wfr = reinterpret_cast<bf16_t*>(smem);
  float* wo = reinterpret_cast<float*>(smem + G_::w_bytes);
  uint4* pair_mask = reinterpret_cast<uint4*>(smem + G_::w_bytes + D * sizeof(float));
  unsigned char* wave_mem = reinterpret_cast<unsigned char*>(pair_mask + 256);

  const int k = g.wblk_k[WM_FWD][blockIdx.x];
  if (k < 0) return;
  const int tid = threadIdx.x, lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int n = lane % 32, h = lane / 32;
  const int grp = lane / G_::LPR, c0 = (lane % G_::LPR) * 8;
  load_weight_fragments<D>(W + static_cast<size_t>(k) * w_stride, wfr);
  fill_pair_masks(pair_mask);
  if (tid < D) wo[tid] = w_out != nullptr ? w_out[static_cast<size_t>(k) * wout_stride + tid] : 0.f;
  __syncthreads();  // the only workgroup barrier: W^k and w_out are in LDS

  const WaveRun run = g.wave_runs[WM_FWD][blockIdx.x * (kBlock / 64) + wave];
  if (run.tile0 >= run.tile1) return;
  unsigned char* my_lds = wave_mem + wave * G_::wave_bytes;
  bf16_t* ot = reinterpret_cast<bf16_t*>(my_lds);  // overlays the row buffer
  stream_tiles<D, D == 128, false>(g, g.went, X, run, my_lds,
                  reinterpret_cast<uint32_t*>(my_lds + G_::xf_bytes), pair_mask, heavy_partial, nullptr,
                  [&](int row0, int nrows, const floatx16 (&agg)[G_::NT]) {
    // Z^T = W^T AGG^T: the rounded aggregate is the B operand as it stands
    floatx16 z[G_::NT];
#pragma unroll
    for (int tj = 0; tj < G_::NT; ++tj)
#pragma unroll
      for (int r = 0; r < 16; ++r) z[tj][r] = 0.f;
    uint4 bq[G_::KS2];
#pragma unroll
    for (int ks2 = 0; ks2 < G_::KS2; ++ks2) {
      float v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = agg[ks2 / 2][8 * (ks2 % 2) + e];
      bq[ks2] = pack8(v);
    }
    // per output tile: all fragments of W first, then the chain of products, so that the
    // products do not wait for one LDS read each
#pragma unroll
    for (int tj = 0; tj < G_::NT; ++tj) {
      uint4 wa[G_::KS2];
#pragma unroll
      for (int ks2 = 0; ks2 < G_::KS2; ++ks2)
        wa[ks2] = *reinterpret_cast<const uint4*>(wfr + ((tj * G_::KS2 + ks2) * 64 + lane) * 8);
#pragma unroll
      for (int ks2 = 0; ks2 < G_::KS2; ++ks2)
        z[tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(wa[ks2]), as_frag(bq[ks2]), z[tj], 0, 0, 0);
    }
    // ReLU, round; lane (n, h) holds features acc_feature(tj, h, r) of row n
    float part = 0.f;
#pragma unroll
    for (int tj = 0; tj < G_::NT; ++tj)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int f0 = acc_feature(tj, 0, 4 * i) + 4 * h;
        uint2 pk;
        pk.x = relu_bf16x2(f32x2_to_bf16x2(z[tj][4 * i], z[tj][4 * i + 1]));
        pk.y = relu_bf16x2(f32x2_to_bf16x2(z[tj][4 * i + 2], z[tj][4 * i + 3]));
        if (w_out != nullptr) {
          const float4 wv = *reinterpret_cast<const float4*>(wo + f0);
          part = fmaf(__uint_as_float(pk.x << 16), wv.x, part);
          part = fmaf(__uint_as_float(pk.x & 0xffff0000u), wv.y, part);
          part = fmaf(__uint_as_float(pk.y << 16), wv.z, part);
          part = fmaf(__uint_as_float(pk.y & 0xffff0000u), wv.w, part);
        }
        *reinterpret_cast<uint2*>(ot + n * G_::PA + f0) = pk;
      }
    // full rows, 16 bytes per lane
    wave_lds_handoff();
#pragma unroll
    for (int u = 0; u < G_::NO; ++u) {
      const int r = u * G_::NG + grp;
      if (r < nrows)
        store_streamed(Y + static_cast<size_t>(row0 + r) * D + c0,
                       *reinterpret_cast<const uint4*>(ot + r * G_::PA + c0));
    }
    wave_lds_handoff();
    if (w_out != nullptr) {  // t[r] = sum_c Y[r, c] * w_out[c]
      part += __shfl_xor(part, 32, 64);
      if (h == 0 && n < nrows) t[row0 + n] = part;
    }
  });
}

// ---------------------------------------------------------------------------
// G_Z of the last hidden layer, formed row by row from the scalar layer's gradient:
//   GZ[i, :] = g_t[i] * w_out^k * [Hcur[i, :] > 0]      (rounded to bf16)
// and the scalar layer's weight gradient, one partial per workgroup:
//   gwout_partial[workgroup, :] = sum_i Hcur[i, :] g_t[i].
// One workgroup per 256-row tile of the narrow decomposition.  The g.num_chunks workgroups
// after those pre-reduce the chunks of the rows with very many neighbours for the
// aggregation A_hat^T G_Z that follows (g is the view of the transposed matrix): they form
// the rows of G_Z they gather on the fly, to the same bits as the rows stored here.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kBlock) void form_gz_last_kernel(
    GraphView g, const bf16_t* __restrict__ Hcur, const float* __restrict__ g_t,
    const float* __restrict__ w_out, int wout_stride, bf16_t* __restrict__ GZ,
    float* __restrict__ gwout_partial, float* __restrict__ heavy_partial) {
  constexpr int LPR = D / 8, RP = kBlock / LPR;  // lanes per row, rows per pass
  __shared__ float red[RP][D + 1];
  static_assert(sizeof(red) >= kBlock * 8 * sizeof(float), "the chunk reduction shares this buffer");
  if (static_cast<int>(blockIdx.x) >= g.num_nblocks) {
    const int ch = blockIdx.x - g.num_nblocks;
    const int kc = g.chunk_part[ch];
    if (kc < 0) return;  // the row's subgraph sits out
    ChunkLastLayerRows<D> rows{Hcur, g_t, {}};
#pragma unroll
    for (int x = 0; x < 8; ++x)
      rows.w[x] = w_out[static_cast<size_t>(kc) * wout_stride + (threadIdx.x % LPR) * 8 + x];
    reduce_chunk<D>(g, rows, heavy_partial, ch, &red[0][0]);
    return;
  }
  const int k = g.nblk_k[blockIdx.x];
  if (k < 0) return;
  const int s = g.nblk_s[blockIdx.x];
  const int rbeg = g.part_rows[k], rend = g.part_rows[k + 1];
  const int rr = threadIdx.x / LPR, c0 = (threadIdx.x % LPR) * 8;
  float wv[8], gacc[8];
#pragma unroll
  for (int x = 0; x < 8; ++x) {
    wv[x] = w_out[static_cast<size_t>(k) * wout_stride + c0 + x];
    gacc[x] = 0.f;
  }
  for (int row0 = rbeg + s * kNarrowRows; row0 < rend; row0 += g.nblk_S[blockIdx.x] * kNarrowRows) {
    const int nrows = min(kNarrowRows, rend - row0);
    for (int r = rr; r < nrows; r += RP) {
      const size_t off = static_cast<size_t>(row0 + r) * D + c0;
      const float gt = g_t[row0 + r];
      float hv[8], out[8];
      unpack8(load_streamed(Hcur + off), hv);
#pragma unroll
      for (int x = 0; x < 8; ++x) {
        out[x] = hv[x] > 0.f ? gt * wv[x] : 0.f;
        gacc[x] = fmaf(hv[x], gt, gacc[x]);
      }
      *reinterpret_cast<uint4*>(GZ + off) = pack8(out);
    }
  }
#pragma unroll
  for (int x = 0; x < 8; ++x) red[rr][c0 + x] = gacc[x];
  __syncthreads();
  if (threadIdx.x < D) {
    float acc = 0.f;
    for (int r = 0; r < RP; ++r) acc += red[r][threadIdx.x];
    gwout_partial[static_cast<size_t>(blockIdx.x) * D + threadIdx.x] = acc;
  }
}

// Positive halves of h select the halves of v (two packed bf16 values each).
__device__ __forceinline__ uint32_t keep_where_positive(uint32_t v, uint32_t h) {
  typedef short i16x2_t __attribute__((ext_vector_type(2)));
  typedef unsigned short u16x2_t __attribute__((ext_vector_type(2)));
  i16x2_t hs;
  __builtin_memcpy(&hs, &h, 4);
  const i16x2_t zero = {0, 0}, one = {1, 1};
  hs = __builtin_elementwise_min(__builtin_elementwise_max(hs, zero), one);  // 1 where h > 0
  u16x2_t m, vv;
  __builtin_memcpy(&m, &hs, 4);
  __builtin_memcpy(&vv, &v, 4);
  vv = vv * m;
  uint32_t r;
  __builtin_memcpy(&r, &vv, 4);
  return r;
}

template <int D>
constexpr size_t bwd_wave_lds() {
  return WG<D>::w_bytes + 256 * sizeof(uint4) + 4 * WG<D>::bwd_wave_bytes;
}

// ---------------------------------------------------------------------------
// Backward of a hidden layer:  G_T = A_hat^T G_Z  (stream_tiles over the transposed
// light stream);  gW partial = sum over the workgroup's rows of Hprev^T G_T;
// G_Hprev = G_T W^T;  then GZ_out = G_Hprev * [Hprev > 0], or, on the embedding
// (TO_EMBED), Adam on E / writing the gradient.
// Width 64, per tile, in the wave's LDS region: G_T (bf16) and Hprev, both transposed to
// [feature][row], feed the weight-gradient product (contraction over the 32 rows).
// Width 128: the rows of G_T (bf16) are stored to a.GT instead and grad_w_wave_kernel
// forms the weight gradient.  The rounded G_T^T in registers is the B operand of
// G_H^T = W G_T^T; the result is staged once more to reach full rows.  Hprev rows of the
// next tile are requested while the current one is finished.
// ---------------------------------------------------------------------------
template <int D, bool TO_EMBED>
__global__ __launch_bounds__(kBlock, 2) void bwd_wave_kernel(GraphView g, BwdArgs a) {
  using G_ = WG<D>;
  constexpr bool GWI = G_::GW_INLINE;
  constexpr bool NEED_HP = GWI || !TO_EMBED;  // Hprev: operand of the weight gradient, ReLU mask
  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* wfr = reinterpret_cast<bf16_t*>(smem);
  uint4* pair_mask = reinterpret_cast<uint4*>(smem + G_::w_bytes);
  unsigned char* wave_mem = reinterpret_cast<unsigned char*>(pair_mask + 256);
  static_assert(!GWI || 4 * G_::bwd_wave_bytes >= 2 * D * D * sizeof(float), "room for the gradient reduction");

  constexpr int WM = TO_EMBED ? WM_EMBED : WM_BWD;
  const int k = g.wblk_k[WM][blockIdx.x];
  if (k < 0) return;
  const AdamStep ad = a.adam.for_part(k);
  const int tid = threadIdx.x, lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int n = lane % 32, h = lane / 32;
  const int grp = lane / G_::LPR, sub = lane % G_::LPR;
  load_weight_fragments_t<D>(a.W + static_cast<size_t>(k) * a.w_stride, wfr);
  fill_pair_masks(pair_mask);
  __syncthreads();

  const bf16_t* GZ = static_cast<const bf16_t*>(a.GZ_in);
  const bf16_t* Hprev = static_cast<const bf16_t*>(a.Hprev);
  const WaveRun run = g.wave_runs[WM][blockIdx.x * (kBlock / 64) + wave];
  unsigned char* R = wave_mem + wave * G_::bwd_wave_bytes;
  const bool need_gh = !(TO_EMBED && a.mode == EMBED_SKIP);
  constexpr int NTW = GWI ? G_::NT : 1;
  floatx16 gw[NTW][NTW];
#pragma unroll
  for (int ta = 0; ta < NTW; ++ta)
#pragma unroll
    for (int tb = 0; tb < NTW; ++tb)
#pragma unroll
      for (int r = 0; r < 16; ++r) gw[ta][tb][r] = 0.f;

  if (run.tile0 < run.tile1) {
    const int rbeg = run.rbeg;
    const int row_end = min(run.rend, rbeg + run.tile1 * RW);
    // rows RPL grp + u (u < RPL) of a tile, features 8 sub .. + 7: what this lane loads of
    // Hprev and what it stores of the result
    constexpr int RPL = RW / G_::NG;
    uint4 hp_raw[NEED_HP ? RPL : 1];
    auto request_hprev = [&](int row0) {
      if (NEED_HP) {
#pragma unroll
        for (int u = 0; u < RPL; ++u) {
          const int r = row0 + RPL * grp + u;
          hp_raw[u] = make_uint4(0u, 0u, 0u, 0u);
          if (r < row_end) hp_raw[u] = load_streamed(Hprev + static_cast<size_t>(r) * D + sub * 8);
        }
      }
    };
    request_hprev(rbeg + run.tile0 * RW);

    stream_tiles<D, false, G_::BWD_LDS_ENTRIES>(g, g.went, GZ, run, R, reinterpret_cast<uint32_t*>(R + G_::region_bytes),
                    pair_mask, a.heavy_partial, R + G_::region_bytes + G_::wts_bytes,
                    [&](int row0, int nrows, const floatx16 (&agg)[G_::NT]) {
      // G_T^T rounded to bf16: B operands of the second product
      uint4 bq[G_::KS2];
#pragma unroll
      for (int ks2 = 0; ks2 < G_::KS2; ++ks2) {
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = agg[ks2 / 2][8 * (ks2 % 2) + e];
        bq[ks2] = pack8(v);
      }
      if constexpr (GWI) {
        static_assert(!GWI || RPL == 4, "four rows per lane group");
        // G_T and Hprev as [feature][row]
        unsigned char* gtl = R;
        unsigned char* hpl = R + D * G_::GP;
#pragma unroll
        for (int ks2 = 0; ks2 < G_::KS2; ++ks2)
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            const int f = feature_of(ks2, 0, 2 * d) + 4 * h;
            const uint32_t w = (&bq[ks2].x)[d];
            *reinterpret_cast<uint16_t*>(gtl + f * G_::GP + n * 2) = static_cast<uint16_t>(w & 0xffffu);
            *reinterpret_cast<uint16_t*>(gtl + (f + 1) * G_::GP + n * 2) = static_cast<uint16_t>(w >> 16);
          }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const uint32_t x0 = (&hp_raw[0].x)[i / 2], x1 = (&hp_raw[1 % RPL].x)[i / 2];
          const uint32_t x2 = (&hp_raw[2 % RPL].x)[i / 2], x3 = (&hp_raw[3 % RPL].x)[i / 2];
          uint2 d;
          d.x = (i % 2 == 0) ? lower_halves(x0, x1) : upper_halves(x0, x1);
          d.y = (i % 2 == 0) ? lower_halves(x2, x3) : upper_halves(x2, x3);
          // 16-byte groups rotated by feature / 8 (LDS banks, as for the row buffer)
          *reinterpret_cast<uint2*>(hpl + (sub * 8 + i) * G_::GP + ((grp / 2 + sub) % 4) * 16 + (grp % 2) * 8) = d;
        }
        wave_lds_handoff();
        // gW[a, b] += sum over the tile's rows of Hprev[row, a] G_T[row, b]
#pragma unroll
        for (int ks = 0; ks < RW / 16; ++ks) {
          bf16x8 af[G_::NT], bf[G_::NT];
#pragma unroll
          for (int t = 0; t < G_::NT; ++t) {
            af[t] = as_frag(*reinterpret_cast<const uint4*>(hpl + (32 * t + n) * G_::GP +
                                                            ((2 * ks + h + (32 * t + n) / 8) % 4) * 16));
            bf[t] = as_frag(*reinterpret_cast<const uint4*>(gtl + (32 * t + n) * G_::GP + (16 * ks + 8 * h) * 2));
          }
#pragma unroll
          for (int ta = 0; ta < NTW; ++ta)
#pragma unroll
            for (int tb = 0; tb < NTW; ++tb)
              gw[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ta], bf[tb], gw[ta][tb], 0, 0, 0);
        }
        wave_lds_handoff();
      } else {
        // the rows of G_T go to memory: lane (n, h) holds, per contraction step, features
        // feature_of(ks2, h, 0..3) and feature_of(ks2, h, 4..7) of row n
        bf16_t* ot = reinterpret_cast<bf16_t*>(R);
#pragma unroll
        for (int ks2 = 0; ks2 < G_::KS2; ++ks2) {
          *reinterpret_cast<uint2*>(ot + n * G_::PA + feature_of(ks2, 0, 0) + 4 * h) =
              make_uint2(bq[ks2].x, bq[ks2].y);
          *reinterpret_cast<uint2*>(ot + n * G_::PA + feature_of(ks2, 0, 4) + 4 * h) =
              make_uint2(bq[ks2].z, bq[ks2].w);
        }
        wave_lds_handoff();
        bf16_t* GT = static_cast<bf16_t*>(a.GT);
#pragma unroll
        for (int u = 0; u < RPL; ++u) {
          const int r = RPL * grp + u;
          if (r < nrows)
            store_streamed(GT + static_cast<size_t>(row0 + r) * D + sub * 8,
                           *reinterpret_cast<const uint4*>(ot + r * G_::PA + sub * 8));
        }
        wave_lds_handoff();
      }
      if (need_gh) {
        // G_H^T = W G_T^T
        floatx16 z[G_::NT];
#pragma unroll
        for (int ta = 0; ta < G_::NT; ++ta)
#pragma unroll
          for (int r = 0; r < 16; ++r) z[ta][r] = 0.f;
#pragma unroll
        for (int ks2 = 0; ks2 < G_::KS2; ++ks2)
#pragma unroll
          for (int ta = 0; ta < G_::NT; ++ta) {
            const bf16x8 wa =
                as_frag(*reinterpret_cast<const uint4*>(wfr + ((ta * G_::KS2 + ks2) * 64 + lane) * 8));
            z[ta] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa, as_frag(bq[ks2]), z[ta], 0, 0, 0);
          }
        if (TO_EMBED) {
          // full fp32 rows through the region (RS rows at a time), then Adam (or the plain
          // gradient)
          float* st = reinterpret_cast<float*>(R);
          constexpr int LR = D / 4;          // lanes per fp32 row
          constexpr int RI = 64 / LR;        // rows per instruction
          constexpr int NQ = G_::RS / RI;    // instructions per pass and tensor
          constexpr int HB = D == 64 ? 4 : 2;  // rows of state requested at once, per lane
          static_assert(NQ % HB == 0, "whole groups of requests");
          const int rr = lane / LR, cc = (lane % LR) * 4;
#pragma unroll
          for (int sp = 0; sp < G_::SP; ++sp) {
            if (n / G_::RS == sp) {
#pragma unroll
              for (int ta = 0; ta < G_::NT; ++ta)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                  *reinterpret_cast<float4*>(st + (n % G_::RS) * G_::PF + acc_feature(ta, 0, 4 * i) + 4 * h) =
                      make_float4(z[ta][4 * i], z[ta][4 * i + 1], z[ta][4 * i + 2], z[ta][4 * i + 3]);
            }
            wave_lds_handoff();
            if (a.mode == EMBED_WRITE_GRAD) {
#pragma unroll
              for (int q = 0; q < NQ; ++q) {
                const int r = sp * G_::RS + q * RI + rr;
                if (r < nrows)
                  *reinterpret_cast<float4*>(a.gE + static_cast<size_t>(row0 + r) * D + cc) =
                      *reinterpret_cast<const float4*>(st + (q * RI + rr) * G_::PF + cc);
              }
            } else {
              // the state of HB * RI rows is requested at once, so that the loads overlap
              float* __restrict__ pE = a.E;
              float* __restrict__ pM = a.mE;
              float* __restrict__ pV = a.vE;
              bf16_t* __restrict__ pB = static_cast<bf16_t*>(a.Eb);
#pragma unroll
              for (int part = 0; part < NQ / HB; ++part) {
                float4 e0[HB], m0[HB], v0[HB];
#pragma unroll
                for (int q = 0; q < HB; ++q) {
                  const int r = sp * G_::RS + (part * HB + q) * RI + rr;
                  const size_t off = static_cast<size_t>(row0 + min(r, nrows - 1)) * D + cc;
                  m0[q] = load_streamed(pM + off);
                  v0[q] = load_streamed(pV + off);
                  e0[q] = load_streamed(pE + off);
                }
#pragma unroll
                for (int q = 0; q < HB; ++q) {
                  const int rl = (part * HB + q) * RI + rr, r = sp * G_::RS + rl;
                  const float4 gq = *reinterpret_cast<const float4*>(st + rl * G_::PF + cc);
                  const size_t off = static_cast<size_t>(row0 + r) * D + cc;
                  const float gv[4] = {gq.x, gq.y, gq.z, gq.w};
                  const float mv[4] = {m0[q].x, m0[q].y, m0[q].z, m0[q].w};
                  const float vv[4] = {v0[q].x, v0[q].y, v0[q].z, v0[q].w};
                  const float ev[4] = {e0[q].x, e0[q].y, e0[q].z, e0[q].w};
                  float mo[4], vo[4], eo[4];
#pragma unroll
                  for (int x = 0; x < 4; ++x) {
                    mo[x] = ad.b1 * mv[x] + (1.f - ad.b1) * gv[x];
                    vo[x] = ad.b2 * vv[x] + (1.f - ad.b2) * gv[x] * gv[x];
                    // v_sqrt_f32 and v_rcp_f32: 1 ulp each
                    const float upd = (mo[x] * ad.inv_bc1) *
                                      __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(vo[x]) * ad.inv_sqrt_bc2 +
                                                            ad.eps);
                    eo[x] = ev[x] - ad.lr * upd;
                  }
                  if (r < nrows) {
                    store_streamed(pM + off, mo[0], mo[1], mo[2], mo[3]);
                    store_streamed(pV + off, vo[0], vo[1], vo[2], vo[3]);
                    store_streamed(pE + off, eo[0], eo[1], eo[2], eo[3]);
                    uint2 eb;
                    eb.x = f32x2_to_bf16x2(eo[0], eo[1]);
                    eb.y = f32x2_to_bf16x2(eo[2], eo[3]);
                    *reinterpret_cast<uint2*>(pB + off) = eb;
                  }
                }
              }
            }
            if (sp + 1 < G_::SP) wave_lds_handoff();  // the next rows overwrite the staging area
          }
        } else {
          // GZ_out = G_Hprev * [Hprev > 0]: full bf16 rows through the region
          bf16_t* ot = reinterpret_cast<bf16_t*>(R);
#pragma unroll
          for (int ta = 0; ta < G_::NT; ++ta)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              uint2 pk;
              pk.x = f32x2_to_bf16x2(z[ta][4 * i], z[ta][4 * i + 1]);
              pk.y = f32x2_to_bf16x2(z[ta][4 * i + 2], z[ta][4 * i + 3]);
              *reinterpret_cast<uint2*>(ot + n * G_::PA + acc_feature(ta, 0, 4 * i) + 4 * h) = pk;
            }
          wave_lds_handoff();
          bf16_t* GZo = static_cast<bf16_t*>(a.GZ_out);
#pragma unroll
          for (int u = 0; u < RPL; ++u) {
            const int r = RPL * grp + u;
            uint4 o = *reinterpret_cast<const uint4*>(ot + r * G_::PA + sub * 8);
            o.x = keep_where_positive(o.x, hp_raw[NEED_HP ? u : 0].x);
            o.y = keep_where_positive(o.y, hp_raw[NEED_HP ? u : 0].y);
            o.z = keep_where_positive(o.z, hp_raw[NEED_HP ? u : 0].z);
            o.w = keep_where_positive(o.w, hp_raw[NEED_HP ? u : 0].w);
            if (r < nrows) store_streamed(GZo + static_cast<size_t>(row0 + r) * D + sub * 8, o);
          }
        }
      }
      wave_lds_handoff();
      request_hprev(row0 + RW);
    });
  }

  if constexpr (GWI) {
    // weight-gradient partial of the workgroup: (wave 0 + wave 2) + (wave 1 + wave 3)
    __syncthreads();
    float* buf = reinterpret_cast<float*>(wave_mem);
    for (int pass = 0; pass < 2; ++pass) {
      if (wave / 2 == pass) {
        float* b = buf + (wave % 2) * D * D;
#pragma unroll
        for (int ta = 0; ta < NTW; ++ta)
#pragma unroll
          for (int tb = 0; tb < NTW; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              float* p = b + acc_feature(ta, h, r) * D + 32 * tb + n;
              *p = pass == 0 ? gw[ta][tb][r] : *p + gw[ta][tb][r];
            }
      }
      __syncthreads();
    }
    float* out = a.gW_partial + static_cast<size_t>(blockIdx.x) * D * D;
    for (int idx = tid; idx < D * D; idx += kBlock) out[idx] = buf[idx] + buf[D * D + idx];
  }
}

// Transposing 8-byte LDS read (ds_read_b64_tr_b16): in every group of 16 lanes, lane 4 r + c
// receives element c (16 bits) of the four 8-byte chunks addressed by lanes r, r + 4, r + 8,
// r + 12 of the group, in that order.
typedef short i16x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ i16x4_t lds_read_transposed(uint32_t addr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4_t*)(uintptr_t)addr);
}
__device__ __forceinline__ bf16x8 frag_of(const i16x4_t& lo, const i16x4_t& hi) {
  uint4 u;
  u.x = (static_cast<uint32_t>(static_cast<uint16_t>(lo[1])) << 16) | static_cast<uint16_t>(lo[0]);
  u.y = (static_cast<uint32_t>(static_cast<uint16_t>(lo[3])) << 16) | static_cast<uint16_t>(lo[2]);
  u.z = (static_cast<uint32_t>(static_cast<uint16_t>(hi[1])) << 16) | static_cast<uint16_t>(hi[0]);
  u.w = (static_cast<uint32_t>(static_cast<uint16_t>(hi[3])) << 16) | static_cast<uint16_t>(hi[2]);
  return as_frag(u);
}

// ---------------------------------------------------------------------------
// Weight gradient of a hidden layer of width 128 (the weight part of Eq. 3's backward), from
// stored rows:  gW partial[workgroup] = sum over the workgroup's rows of Hprev[row, :]^T GT[row, :].
// A decomposition of its own (WM_GRADW: a wavefront owns a run of 32-row tiles, one
// workgroup per compute unit).  One wavefront per SIMD (the 128 x 128
// accumulator is 256 registers per lane).  With a single wavefront per SIMD nothing hides a
// memory round trip but the wavefront's own requests, so the rows travel straight into a
// wave-private LDS ring of two tiles (32 rows of both matrices each) and up to two tiles are
// on their way while one is multiplied.  A tile sits in LDS row by row: the 16-byte pieces of
// rows 4 i .. 4 i + 3 fill 1 KB, piece p of row r at position p ^ 2 (r % 4), which spreads the
// four rows of a transposing read over all banks.  Fragments: lane (n, h) of an operand needs
// 8 consecutive rows of feature 32 t + n -- two transposing reads whose source lane
// s = 4 j + r' (of the 16-lane group g) points at row (8 (g / 2) + j [+ 4]) of the contraction
// step, features 32 t + 16 (g % 2) + 4 r' .. + 3.
// ---------------------------------------------------------------------------
template <int D>
constexpr size_t grad_w_lds() {
  return 4 * 2 * 2 * static_cast<size_t>(RW) * D * 2;  // 4 wavefronts x 2 tiles x 2 matrices
}

template <int D>
__global__ __launch_bounds__(kBlock, 1) void grad_w_wave_kernel(GraphView g, const bf16_t* __restrict__ Hprev,
                                                                const bf16_t* __restrict__ GT,
                                                                float* __restrict__ gW_partial) {
  using G_ = WG<D>;
  static_assert(D == 128, "16 lanes per row of 16-byte pieces");
  static_assert(grad_w_lds<D>() >= 2 * static_cast<size_t>(D) * D * sizeof(float), "room for the reduction");
  constexpr uint32_t kTile = RW * D * 2;  // bytes of one matrix's tile
  extern __shared__ __align__(16) unsigned char smem[];
  const int k = g.wblk_k[WM_GRADW][blockIdx.x];
  if (k < 0) return;
  const int tid = threadIdx.x, lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int n = lane % 32, h = lane / 32;
  const WaveRun run = g.wave_runs[WM_GRADW][blockIdx.x * (kBlock / 64) + wave];
  unsigned char* ring = smem + wave * (4 * kTile);
  const uint32_t ring_lds = lds_offset(ring);
  floatx16 acc[G_::NT][G_::NT];
#pragma unroll
  for (int ta = 0; ta < G_::NT; ++ta)
#pragma unroll
    for (int tb = 0; tb < G_::NT; ++tb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[ta][tb][r] = 0.f;

  if (run.tile0 < run.tile1) {
    const int rbeg = run.rbeg;
    const int row_end = min(run.rend, rbeg + run.tile1 * RW);  // > rbeg + run.tile0 * RW
    // what this lane copies in every request: row (lane / 16) of a group of four, piece
    // (lane % 16) ^ 2 (lane / 16) of it
    const int copy_row = lane / 16;
    const int copy_off = ((lane % 16) ^ (2 * copy_row)) * 8;  // in bf16 elements
    // rows past the end are read from the last valid row and zeroed in LDS afterwards
    auto request = [&](int tau, int slot) {
      const int row0 = rbeg + tau * RW;
      const uint32_t base = ring_lds + slot * (2 * kTile);
#pragma unroll
      for (int i = 0; i < RW / 4; ++i) {
        const size_t r = static_cast<size_t>(min(row0 + 4 * i + copy_row, row_end - 1));
        load_to_lds_16(Hprev + r * D + copy_off, base + i * 1024);
        load_to_lds_16(GT + r * D + copy_off, base + kTile + i * 1024);
      }
    };
    // byte offset inside a tile of this lane's chunk in a transposing read of feature tile t,
    // contraction step ks, row half q
    const int g16 = lane / 16, s16 = lane % 16, jj = s16 / 4, rr = s16 % 4;
    auto chunk = [&](int t, int ks, int q) -> uint32_t {
      const int piece = (4 * t + 2 * (g16 % 2) + rr / 2) ^ (2 * jj);
      return static_cast<uint32_t>((4 * ks + 2 * (g16 / 2) + q) * 1024 + jj * 256 + piece * 16 + (rr % 2) * 8);
    };
    request(run.tile0, 0);
    if (run.tile0 + 1 < run.tile1) request(run.tile0 + 1, 1);
    for (int tau = run.tile0; tau < run.tile1; ++tau) {
      const int slot = (tau - run.tile0) & 1;
      const uint32_t base = ring_lds + slot * (2 * kTile);
      // tile tau has landed once at most the next tile's 2 * RW / 4 copies are outstanding
      if (tau + 1 < run.tile1) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      static_assert(2 * (RW / 4) == 16, "the wait above counts the copies of one tile");
      const int nrows = min(RW, row_end - (rbeg + tau * RW));
      if (nrows < RW) {  // the subgraph's last tile: rows past its end count as zero
        for (int r = nrows + lane / 16; r < RW; r += 4)
          *reinterpret_cast<uint4*>(ring + slot * (2 * kTile) + (r / 4) * 1024 + (r % 4) * 256 + (lane % 16) * 16) =
              make_uint4(0u, 0u, 0u, 0u);
      }
      wave_lds_handoff();
      bf16x8 af[G_::NT][RW / 16], bf[G_::NT][RW / 16];
#pragma unroll
      for (int ks = 0; ks < RW / 16; ++ks)
#pragma unroll
        for (int t = 0; t < G_::NT; ++t) {
          af[t][ks] = frag_of(lds_read_transposed(base + chunk(t, ks, 0)), lds_read_transposed(base + chunk(t, ks, 1)));
          bf[t][ks] = frag_of(lds_read_transposed(base + kTile + chunk(t, ks, 0)),
                              lds_read_transposed(base + kTile + chunk(t, ks, 1)));
        }
      // every fragment is in registers: the slot may receive the tile after the next
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      if (tau + 2 < run.tile1) request(tau + 2, slot);
#pragma unroll
      for (int ks = 0; ks < RW / 16; ++ks)
#pragma unroll
        for (int ta = 0; ta < G_::NT; ++ta)
#pragma unroll
          for (int tb = 0; tb < G_::NT; ++tb)
            acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ta][ks], bf[tb][ks], acc[ta][tb], 0, 0, 0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }

  // ((wave 0 + wave 1) + wave 2) + wave 3: the running sum travels through two halves of the
  // LDS in turn, so a wavefront first reads all of what the one before wrote (nothing it
  // writes lies between its reads) and then writes all of its own
  float* buf = reinterpret_cast<float*>(smem);
  __syncthreads();  // every ring is done with
#pragma unroll 1
  for (int w = 0; w < kBlock / 64; ++w) {
    if (wave == w) {
      const float* src = buf + ((w - 1) & 1) * (D * D) + n;
      float* dst = buf + (w & 1) * (D * D) + n;
      if (w == 0) {
#pragma unroll
        for (int ta = 0; ta < G_::NT; ++ta)
#pragma unroll
          for (int tb = 0; tb < G_::NT; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) dst[acc_feature(ta, h, r) * D + 32 * tb] = acc[ta][tb][r];
      } else {
#pragma unroll
        for (int ta = 0; ta < G_::NT; ++ta)
#pragma unroll
          for (int tb = 0; tb < G_::NT; ++tb) {
            float sum[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) sum[r] = src[acc_feature(ta, h, r) * D + 32 * tb];
#pragma unroll
            for (int r = 0; r < 16; ++r) dst[acc_feature(ta, h, r) * D + 32 * tb] = sum[r] + acc[ta][tb][r];
            __builtin_amdgcn_sched_barrier(0);  // 16 reads at a time: all 256 at once do not fit the registers
          }
      }
    }
    __syncthreads();
  }
  buf += ((kBlock / 64 - 1) & 1) * (D * D);  // where the last wavefront wrote
  float* out = gW_partial + static_cast<size_t>(blockIdx.x) * D * D;
  for (int idx = tid; idx < D * D; idx += kBlock) out[idx] = buf[idx];
}

template <typename K>
void allow_lds(K kernel, size_t bytes) {
  if (bytes > 48 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
}

}  // namespace

void launch_form_gz_last(const Launch& ln, int D, const GraphView& g, const BwdArgs& a) {
  ln.begin(KK_FORM_GZ);
  if (D == 64)
    form_gz_last_kernel<64><<<g.num_nblocks + g.num_chunks, kBlock, 0, ln.st>>>(
        g, static_cast<const bf16_t*>(a.Hcur), a.g_t, a.w_out, a.wout_stride, static_cast<bf16_t*>(a.GZ_last),
        a.gwout_partial, a.heavy_partial);
  else if (D == 128)
    form_gz_last_kernel<128><<<g.num_nblocks + g.num_chunks, kBlock, 0, ln.st>>>(
        g, static_cast<const bf16_t*>(a.Hcur), a.g_t, a.w_out, a.wout_stride, static_cast<bf16_t*>(a.GZ_last),
        a.gwout_partial, a.heavy_partial);
  ln.end(KK_FORM_GZ);
}

template <int D>
static void bwd_wave_t(const Launch& ln, bool to_embed, const GraphView& gt, const BwdArgs& a) {
  const int kind = to_embed ? KK_BWD_EMBED : KK_BWD_HIDDEN;
  ln.begin(kind);
  if (to_embed) {
    allow_lds(bwd_wave_kernel<D, true>, bwd_wave_lds<D>());
    bwd_wave_kernel<D, true><<<gt.num_wblocks[WM_EMBED], kBlock, bwd_wave_lds<D>(), ln.st>>>(gt, a);
  } else {
    allow_lds(bwd_wave_kernel<D, false>, bwd_wave_lds<D>());
    bwd_wave_kernel<D, false><<<gt.num_wblocks[WM_BWD], kBlock, bwd_wave_lds<D>(), ln.st>>>(gt, a);
  }
  ln.end(kind);
}

void launch_bwd_hidden_wave(const Launch& ln, int D, bool to_embed, const GraphView& gt, const BwdArgs& a) {
  if (D == 64) {
    bwd_wave_t<64>(ln, to_embed, gt, a);
  } else if (D == 128) {
    bwd_wave_t<128>(ln, to_embed, gt, a);
    // the weight gradient from the stored rows of G_T
    allow_lds(grad_w_wave_kernel<128>, grad_w_lds<128>());
    ln.begin(KK_GRAD_W);
    grad_w_wave_kernel<128><<<gt.num_wblocks[WM_GRADW], kBlock, grad_w_lds<128>(), ln.st>>>(
        gt, static_cast<const bf16_t*>(a.Hprev), static_cast<const bf16_t*>(a.GT), a.gW_partial);
    ln.end(KK_GRAD_W);
  }
}

void launch_fwd_hidden_wave(const Launch& ln, int D, const GraphView& g, const void* X, const float* W,
                            int w_stride, void* Y, const float* w_out, int wout_stride, float* t,
                            float* heavy_partial) {
  ln.begin(KK_FWD_HIDDEN);
  if (D == 64) {
    allow_lds(fwd_wave_kernel<64>, fwd_wave_lds<64>());
    fwd_wave_kernel<64><<<g.num_wblocks[WM_FWD], kBlock, fwd_wave_lds<64>(), ln.st>>>(
        g, static_cast<const bf16_t*>(X), W, w_stride, static_cast<bf16_t*>(Y), w_out, wout_stride, t,
        heavy_partial);
  } else if (D == 128) {
    allow_lds(fwd_wave_kernel<128>, fwd_wave_lds<128>());
    fwd_wave_kernel<128><<<g.num_wblocks[WM_FWD], kBlock, fwd_wave_lds<128>(), ln.st>>>(
        g, static_cast<const bf16_t*>(X), W, w_stride, static_cast<bf16_t*>(Y), w_out, wout_stride, t,
        heavy_partial);
  }
  ln.end(KK_FWD_HIDDEN);
}

}  // namespace gco
