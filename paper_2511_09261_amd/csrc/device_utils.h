// Small device helpers: bf16 storage, 16-byte vector access, wavefront reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gco {

typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t h) {
  return __uint_as_float(static_cast<uint32_t>(h) << 16);
}

// Round to nearest, ties to even (IEEE 754 roundTiesToEven on the upper 16 bits).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  const __bf16 b = static_cast<__bf16>(f);  // round to nearest even (v_cvt_pk_bf16_f32)
  bf16_t u;
  __builtin_memcpy(&u, &b, 2);
  return u;
}

// Two fp32 values rounded to bf16 in one word (a in the lower half).
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float a, float b) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {a, b};
  const bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
  uint32_t u;
  __builtin_memcpy(&u, &r, 4);
  return u;
}

// max(x, 0) on two packed bf16 values: a negative bf16 is a negative 16-bit integer.
__device__ __forceinline__ uint32_t relu_bf16x2(uint32_t u) {
  typedef short i16x2_t __attribute__((ext_vector_type(2)));
  i16x2_t s;
  __builtin_memcpy(&s, &u, 4);
  const i16x2_t zero = {0, 0};
  s = __builtin_elementwise_max(s, zero);
  __builtin_memcpy(&u, &s, 4);
  return u;
}

// Storage traits: how a feature row is kept in HBM.
template <typename T>
struct Store;

template <>
struct Store<float> {
  static constexpr int VEC = 4;  // elements per 16-byte access
  static __device__ __forceinline__ void load(const float* p, float (&v)[4]) {
    const float4 x = *reinterpret_cast<const float4*>(p);
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
  static __device__ __forceinline__ float get(const float* p) { return *p; }
  static __device__ __forceinline__ void put(float* p, float x) { *p = x; }
  static __device__ __forceinline__ float as_stored(float x) { return x; }
};

template <>
struct Store<bf16_t> {
  static constexpr int VEC = 8;
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
    const uint4 x = *reinterpret_cast<const uint4*>(p);
    v[0] = __uint_as_float(x.x << 16); v[1] = __uint_as_float(x.x & 0xffff0000u);
    v[2] = __uint_as_float(x.y << 16); v[3] = __uint_as_float(x.y & 0xffff0000u);
    v[4] = __uint_as_float(x.z << 16); v[5] = __uint_as_float(x.z & 0xffff0000u);
    v[6] = __uint_as_float(x.w << 16); v[7] = __uint_as_float(x.w & 0xffff0000u);
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
    uint4 x;
    x.x = f32x2_to_bf16x2(v[0], v[1]);
    x.y = f32x2_to_bf16x2(v[2], v[3]);
    x.z = f32x2_to_bf16x2(v[4], v[5]);
    x.w = f32x2_to_bf16x2(v[6], v[7]);
    *reinterpret_cast<uint4*>(p) = x;
  }
  static __device__ __forceinline__ float get(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void put(bf16_t* p, float x) { *p = f32_to_bf16(x); }
  static __device__ __forceinline__ float as_stored(float x) { return bf16_to_f32(f32_to_bf16(x)); }
};

// Between LDS writes of some lanes of a wavefront and LDS reads of the same locations by
// other lanes of that wavefront: the hardware executes a wavefront's LDS operations in
// program order, so no instruction is needed, but the compiler has to be told that the
// lanes communicate (otherwise it may forward a lane's own earlier store to its load).
__device__ __forceinline__ void wave_lds_handoff() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Sum over the 64 lanes of a wavefront in a fixed butterfly order; every lane
// ends with the total.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

}  // namespace gco
