// Shared device-side helpers and the launch-parameter block of the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/oomb.h"

namespace oomb {

// Everything a kernel needs to find its operands (paper notation, Sec. 4.2).
struct Params {
  int32_t Hq, Hkv, G, D, P, C, m;
  int64_t N, n, n_past;
  float sm_scale;
  int64_t pool_page_stride, pool_head_stride, pool_tok_stride;
  int64_t q_tok_stride, q_head_stride;
  const void* q;
  const void* k_pool;
  const void* v_pool;
  const int32_t* page_table;
  const int32_t* sel;        // NULL = dense
  const int32_t* sel_count;
  int32_t sel_stride;
  void* o;
  float* lse;
  const void* d_o;
  void* d_q;
  void* dk_pool;
  void* dv_pool;
  float* delta;              // [Hq][C], workspace
  int32_t grad_is_bf16;
  uint32_t g_magic;          // ceil(2^32 / G): row / G == umulhi(row, g_magic) for row < 2^32 / G, G > 1
};

typedef uint16_t bf16_t;  // raw bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round to nearest even; inputs are finite in every caller except the masked
// -inf cases, which never reach a store
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Brackets a kernel launch with HIP events when benchmark profiling is enabled
// (oomb_profile_enable); does nothing otherwise.
class ProfScope {
 public:
  ProfScope(const char* name, hipStream_t st);
  ~ProfScope();
 private:
  hipStream_t stream_;
  int slot_;
  hipEvent_t start_;
};

// row-space index -> chunk token (row / G) without an integer division
__device__ __forceinline__ uint32_t div_g(const Params& p, uint32_t r) {
  return p.G == 1 ? r : __umulhi(r, p.g_magic);
}

__device__ __forceinline__ int32_t list_len(const Params& p, int g) {
  return p.sel ? p.sel_count[g] : (int32_t)p.n;
}
__device__ __forceinline__ int32_t list_at(const Params& p, int g, int32_t j) {
  return p.sel ? p.sel[(int64_t)g * p.sel_stride + j] : j;
}

}  // namespace oomb
