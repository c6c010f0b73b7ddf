// What plain streaming kernels reach on the device the library runs on: the yardstick the
// benchmark holds the training kernels against, next to the published HBM figure.
//   kind 0  read-only      (one array in)
//   kind 1  copy           (one array in, one out)
//   kind 2  update in place of three arrays (the access pattern of Adam on the
//           embeddings: E, m, v read and written once each)
// 16 bytes per lane, four (kind 2: two) accesses in flight per lane and array, non-temporal
// loads and stores, grid-stride loop.
#include <hip/hip_runtime.h>

#include "gco.h"
#include "gco_internal.h"

namespace gco {
namespace {

typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <int U>
__global__ __launch_bounds__(kBlock) void probe_read_kernel(const f32x4_t* __restrict__ a, float* __restrict__ sink,
                                                            size_t n4) {
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
  for (size_t i = static_cast<size_t>(blockIdx.x) * kBlock * U + threadIdx.x; i + (U - 1) * kBlock < n4;
       i += static_cast<size_t>(gridDim.x) * kBlock * U) {
    f32x4_t v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(a + i + u * kBlock);
#pragma unroll
    for (int u = 0; u < U; ++u) acc += v[u];
  }
  if (acc.x + acc.y + acc.z + acc.w == 12345.678f) sink[0] = 1.f;  // keeps the loads alive
}

template <int U>
__global__ __launch_bounds__(kBlock) void probe_copy_kernel(const f32x4_t* __restrict__ a, f32x4_t* __restrict__ b,
                                                            size_t n4) {
  for (size_t i = static_cast<size_t>(blockIdx.x) * kBlock * U + threadIdx.x; i + (U - 1) * kBlock < n4;
       i += static_cast<size_t>(gridDim.x) * kBlock * U) {
    f32x4_t v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(a + i + u * kBlock);
#pragma unroll
    for (int u = 0; u < U; ++u) __builtin_nontemporal_store(v[u], b + i + u * kBlock);
  }
}

template <int U>
__global__ __launch_bounds__(kBlock) void probe_update_kernel(f32x4_t* __restrict__ e, f32x4_t* __restrict__ m,
                                                              f32x4_t* __restrict__ v, size_t n4) {
  for (size_t i = static_cast<size_t>(blockIdx.x) * kBlock * U + threadIdx.x; i + (U - 1) * kBlock < n4;
       i += static_cast<size_t>(gridDim.x) * kBlock * U) {
    f32x4_t ev[U], mv[U], vv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      ev[u] = __builtin_nontemporal_load(e + i + u * kBlock);
      mv[u] = __builtin_nontemporal_load(m + i + u * kBlock);
      vv[u] = __builtin_nontemporal_load(v + i + u * kBlock);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      mv[u] = 0.9f * mv[u] + 0.1f * ev[u];
      vv[u] = 0.999f * vv[u] + 0.001f * ev[u] * ev[u];
      ev[u] = ev[u] - 0.001f * mv[u];
      __builtin_nontemporal_store(ev[u], e + i + u * kBlock);
      __builtin_nontemporal_store(mv[u], m + i + u * kBlock);
      __builtin_nontemporal_store(vv[u], v + i + u * kBlock);
    }
  }
}

}  // namespace
}  // namespace gco

extern "C" int gco_stream_probe(int32_t kind, size_t bytes_per_array, int32_t repeats, double* gbytes_per_s) {
  using namespace gco;
  if (kind < 0 || kind > 2 || repeats < 1 || !gbytes_per_s || bytes_per_array < (1u << 20)) return GCO_EINVAL;
  const size_t n4 = bytes_per_array / 16;
  const size_t bytes = n4 * 16;
  const int arrays = kind == 0 ? 1 : (kind == 1 ? 2 : 3);
  f32x4_t* buf[3] = {nullptr, nullptr, nullptr};
  float* sink = nullptr;
  hipEvent_t t0 = nullptr, t1 = nullptr;
  int rc = GCO_OK;
  auto fail = [&](int code) { rc = code; };
  for (int q = 0; q < arrays && rc == GCO_OK; ++q)
    if (hipMalloc(&buf[q], bytes) != hipSuccess || hipMemset(buf[q], 0, bytes) != hipSuccess) fail(GCO_ENOMEM);
  if (rc == GCO_OK && hipMalloc(&sink, sizeof(float)) != hipSuccess) fail(GCO_ENOMEM);
  if (rc == GCO_OK && (hipEventCreate(&t0) != hipSuccess || hipEventCreate(&t1) != hipSuccess)) fail(GCO_EDEVICE);
  if (rc == GCO_OK) {
    const int grid = 16384;
    auto launch = [&]() {
      if (kind == 0) probe_read_kernel<4><<<grid, kBlock>>>(buf[0], sink, n4);
      else if (kind == 1) probe_copy_kernel<4><<<grid, kBlock>>>(buf[0], buf[1], n4);
      else probe_update_kernel<4><<<grid, kBlock>>>(buf[0], buf[1], buf[2], n4);
    };
    launch();  // warm-up
    (void)hipEventRecord(t0, nullptr);
    for (int r = 0; r < repeats; ++r) launch();
    (void)hipEventRecord(t1, nullptr);
    float ms = 0.f;
    if (hipEventSynchronize(t1) != hipSuccess || hipEventElapsedTime(&ms, t0, t1) != hipSuccess || !(ms > 0.f)) {
      fail(GCO_EDEVICE);
    } else {
      const double moved = static_cast<double>(bytes) * (kind == 0 ? 1 : (kind == 1 ? 2 : 6)) * repeats;
      *gbytes_per_s = moved / (static_cast<double>(ms) * 1e-3) / 1e9;
    }
  }
  if (t0) (void)hipEventDestroy(t0);
  if (t1) (void)hipEventDestroy(t1);
  for (int q = 0; q < 3; ++q)
    if (buf[q]) (void)hipFree(buf[q]);
  if (sink) (void)hipFree(sink);
  (void)hipGetLastError();
  return rc;
}
