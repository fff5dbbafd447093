// Shared device-side helpers and the launch-parameter block of the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/oomb.h"
#include "../../include/oomb_bench.h"

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
  // One page list per (KV head, query page) (Sec. 4.2, retrieval by votes): sel is [Hkv][m][sel_stride],
  // sel_count [Hkv][m]; list id = g * m + query page.  The maps below are built on the device by
  // qp_prepare from the lists, in the caller's workspace.
  int32_t qp;                // 0: one list per KV head (list id = g)
  int32_t un_stride;         // row stride of un_list / un_pbase / un_ns; inv_off rows are un_stride + 1 long
  int32_t max_units;         // row stride of units
  const int32_t* qp_slot;    // [Hkv][m][sel_stride]: position of each list entry in the union list
  const int32_t* un_list;    // [Hkv][un_stride]: union of the lists of a KV head, ascending ("owned" pages)
  const int32_t* un_count;   // [Hkv]
  const int32_t* inv_off;    // [Hkv][un_stride + 1]: CSR offsets into inv_qp
  const int32_t* inv_qp;     // [Hkv][m * sel_stride]: the query pages whose list holds a union entry, ascending
  const int4* units;         // [Hkv][max_units] dK/dV work units: (union entry, first inverse-list index,
                             //   number of query pages, partial slot or -1 = straight into the pool)
  const int32_t* unit_count; // [Hkv]
  const int32_t* un_pbase;   // [Hkv][un_stride]: first partial slot of a union entry cut into slices, else -1
  const int32_t* un_ns;      // [Hkv][un_stride]: number of slices
  const int32_t* multi_list; // [Hkv][max_multi]: the union entries that are cut into slices
  const int32_t* multi_count;// [Hkv]
  int32_t max_multi;
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

// A kernel's dynamic-LDS limit is a per-device function attribute: it is raised once on every device
// the kernel is launched on, from whichever thread gets there first (implemented in profile.hip).
struct DeviceOnce {
  static constexpr int MAX_DEVICES = 64;
  unsigned char done[MAX_DEVICES] = {};
};
hipError_t ensure_max_dynamic_lds(DeviceOnce& once, const void* kernel, int bytes);

// row-space index -> chunk token (row / G) without an integer division
__device__ __forceinline__ uint32_t div_g(const Params& p, uint32_t r) {
  return p.G == 1 ? r : __umulhi(r, p.g_magic);
}

// Page lists.  List id `lid`: g with one list per KV head, g * m + query page otherwise.
__device__ __forceinline__ int32_t list_len(const Params& p, int lid) {
  return p.sel ? p.sel_count[lid] : (int32_t)p.n;
}
__device__ __forceinline__ int32_t list_at(const Params& p, int lid, int32_t j) {
  return p.sel ? p.sel[(int64_t)lid * p.sel_stride + j] : j;
}
__device__ __forceinline__ int list_id(const Params& p, int g, int i) {
  return p.qp ? g * p.m + i / p.P : g;
}
// Pages of KV head g that some row attends ("owned" by one dK/dV workgroup each): its list, or the
// union of its per-query-page lists.
__device__ __forceinline__ int32_t owned_len(const Params& p, int g) {
  return p.qp ? p.un_count[g] : list_len(p, g);
}
__device__ __forceinline__ int32_t owned_at(const Params& p, int g, int32_t j) {
  return p.qp ? p.un_list[(int64_t)g * p.un_stride + j] : list_at(p, g, j);
}

}  // namespace oomb
