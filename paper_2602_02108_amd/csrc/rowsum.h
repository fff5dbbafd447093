// Sequential fp32 row sums with 16-byte loads, shared by the page scorer and the paged manager
// (paper Sec. 4.2: a key page is represented by the mean of its keys).  The additions stay in
// token order with one rounding each, so every user produces the same bits.
#pragma once
#include "common.h"

#pragma clang fp contract(off)

namespace oomb {

template <typename T> struct Vec16;  // one 16-byte load worth of elements
template <> struct Vec16<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
  }
};

// 16 bytes, optionally with a non-temporal load
template <bool STREAM> __device__ __forceinline__ uint4 load16(const void* ptr) {
  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
  if (STREAM) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(ptr));
    return make_uint4(v.x, v.y, v.z, v.w);
  }
  return *reinterpret_cast<const uint4*>(ptr);
}

// Left-to-right sum of `count` rows (row stride `stride` elements) of the VEC
// elements this lane owns.  Loads are issued U at a time, adds stay in order.
// STREAM: the rows are read once and not again soon (the whole key history behind the page scorer):
// non-temporal loads, which neither displace what the next kernels need from the caches nor wait for
// an allocation there (page scoring at the 1M-token benchmark shape: 5.0 -> 6.2 TB/s).
template <typename T, int U, bool STREAM = false>
__device__ __forceinline__ void seq_row_sum(const T* base, int64_t stride, int count, float* acc) {
  constexpr int VEC = Vec16<T>::N;
#pragma unroll
  for (int v = 0; v < VEC; ++v) acc[v] = 0.0f;
  int t = 0;
  for (; t + U <= count; t += U) {
    uint4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = load16<STREAM>(base + (int64_t)(t + u) * stride);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float f[VEC];
      Vec16<T>::unpack(r[u], f);
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[v] = __fadd_rn(acc[v], f[v]);
    }
  }
  for (; t < count; ++t) {
    const uint4 r = load16<STREAM>(base + (int64_t)t * stride);
    float f[VEC];
    Vec16<T>::unpack(r, f);
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = __fadd_rn(acc[v], f[v]);
  }
}

}  // namespace oomb
