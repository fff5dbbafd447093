// Building blocks of the bf16 MFMA kernels (gfx950, wave64): vector types, LDS
// tile layouts and the global -> LDS tile movers.  Page size 128, head dim 128.
//
// MFMA used everywhere: v_mfma_f32_32x32x16_bf16, D(32x32) += A(32x16) * B(16x32).
//   A operand: lane l holds A[l % 32][8 * (l / 32) + 0..7]
//   B operand: lane l holds B[8 * (l / 32) + 0..7][l % 32]
//   C/D:       lane l, register r holds C[8 * (r / 4) + 4 * (l / 32) + r % 4][l % 32]
//
// LDS tiles are 128 rows x 256 bytes (16 granules of 16 bytes).  Granule c of
// row r is stored at granule position c ^ (r & 15), which makes both the
// row-per-lane 16-byte operand reads and the row-contiguous writes free of bank
// conflicts.
//   "natural" tile:    row = token, granule c = elements 8c .. 8c+7 of the head dim.
//   "transposed" tile: row = head-dim index d; granule o = 2 * u + hh holds the
//                      eight tokens 16u + 4hh + {0,1,2,3, 8,9,10,11}; this is the
//                      token order in which a lane of C-layout half hh holds the
//                      rows of a 32x32 accumulator block, so a probability block
//                      can feed the next MFMA without any cross-lane movement.
#pragma once
#include "common.h"

namespace oomb {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int TP = 128;                    // tokens per page (tile rows)
constexpr int HD = 128;                    // head dim
constexpr int TILE_BYTES = TP * HD * 2;    // 32 KiB

__device__ __forceinline__ uint32_t pack2_bf16(float a, float b) {
  f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ f32x16 mfma32(const bf16x8& a, const bf16x8& b, const f32x16& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// byte offset of granule c of row r inside a swizzled tile
__device__ __forceinline__ int tile_off(int r, int c) { return (r * 16 + (c ^ (r & 15))) * 16; }

__device__ __forceinline__ uint4 lds_read16(const unsigned char* tile, int r, int c) {
  return *reinterpret_cast<const uint4*>(tile + tile_off(r, c));
}

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(1))) const void* glb_void_ptr;

// s_waitcnt vmcnt(0): every outstanding vector-memory operation of this wave,
// the direct global -> LDS loads included, has completed.
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// One wave moves 16 rows (four 1 KiB chunks) of a natural tile straight from
// global memory into LDS (global_load_lds_dwordx4: lane l writes 16 bytes at
// LDS base + 16 l).  Lane l of a chunk lands at granule position l % 16 of row
// l / 16, so it fetches the source granule that the swizzle maps there.
// row0 must be a multiple of 16.  Completion: wait_vmem() + barrier.
__device__ __forceinline__ void natural_rows_to_lds(const bf16_t* base, int64_t tok_stride, unsigned char* tile,
                                                    int row0, int lane) {
  // address = wave-uniform 64-bit base + 32-bit per-lane offset, so that nothing
  // 64-bit and lane-dependent has to be kept in registers across the main loop
  const uint32_t ts_bytes = (uint32_t)tok_stride * 2u;
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    const uint32_t lrow = 4 * x + (lane >> 4);
    const uint32_t c = (lane & 15) ^ (lrow & 15);
    const char* sbase = reinterpret_cast<const char*>(base + (int64_t)row0 * tok_stride);
    const char* src = sbase + (lrow * ts_bytes + c * 16u);
    __builtin_amdgcn_global_load_lds((glb_void_ptr)src, (lds_void_ptr)(tile + (row0 + 4 * x) * 256), 16, 0, 0);
  }
}

// ---- natural tile: 128 tokens x 128 dims from a (page, head) slab ------------
// NT threads cooperate; each holds 2048 / NT granules in registers between the
// global load and the LDS store.
template <int NT> struct NaturalStage {
  static constexpr int N = 2048 / NT;
  uint4 r[N];
  __device__ __forceinline__ void load(const bf16_t* base, int64_t tok_stride, int tid) {
#pragma unroll
    for (int x = 0; x < N; ++x) {
      const int gi = tid + NT * x;
      r[x] = *reinterpret_cast<const uint4*>(base + (int64_t)(gi >> 4) * tok_stride + (gi & 15) * 8);
    }
  }
  __device__ __forceinline__ void store(unsigned char* tile, int tid) const {
#pragma unroll
    for (int x = 0; x < N; ++x) {
      const int gi = tid + NT * x;
      *reinterpret_cast<uint4*>(tile + tile_off(gi >> 4, gi & 15)) = r[x];
    }
  }
};

// ---- transposed tile -----------------------------------------------------------
// Each wave moves 16 / NW octets; lane l owns head-dim columns 2l, 2l+1 and
// loads one dword per token (a full 256-byte row per wave instruction).
template <int NW> struct TransposedStage {
  static constexpr int OCT = 16 / NW;
  uint32_t r[OCT][8];
  __device__ __forceinline__ void load(const bf16_t* base, int64_t tok_stride, int wave, int lane) {
#pragma unroll
    for (int x = 0; x < OCT; ++x) {
      const int o = wave * OCT + x, u = o >> 1, hh = o & 1;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int tok = 16 * u + 4 * hh + (e & 3) + 8 * (e >> 2);
        r[x][e] = *reinterpret_cast<const uint32_t*>(base + (int64_t)tok * tok_stride + 2 * lane);
      }
    }
  }
  __device__ __forceinline__ void store(unsigned char* tile, int wave, int lane) const {
#pragma unroll
    for (int x = 0; x < OCT; ++x) {
      const int o = wave * OCT + x;
      uint4 lo, hi;
      lo.x = __builtin_amdgcn_perm(r[x][1], r[x][0], 0x05040100u);
      lo.y = __builtin_amdgcn_perm(r[x][3], r[x][2], 0x05040100u);
      lo.z = __builtin_amdgcn_perm(r[x][5], r[x][4], 0x05040100u);
      lo.w = __builtin_amdgcn_perm(r[x][7], r[x][6], 0x05040100u);
      hi.x = __builtin_amdgcn_perm(r[x][1], r[x][0], 0x07060302u);
      hi.y = __builtin_amdgcn_perm(r[x][3], r[x][2], 0x07060302u);
      hi.z = __builtin_amdgcn_perm(r[x][5], r[x][4], 0x07060302u);
      hi.w = __builtin_amdgcn_perm(r[x][7], r[x][6], 0x07060302u);
      *reinterpret_cast<uint4*>(tile + tile_off(2 * lane, o)) = lo;
      *reinterpret_cast<uint4*>(tile + tile_off(2 * lane + 1, o)) = hi;
    }
  }
};

// Page list entries held in registers, 64 per window, two windows deep: lane j of a
// window holds the logical page id of list entry base + j and its physical page.
// The main loops read them with v_readlane, so no iteration waits for a chain of
// dependent memory loads (selection list -> page table); the next window is
// fetched while the current one is consumed.
struct PageWindow {
  int32_t l_cur, p_cur, l_nxt, p_nxt;
  int32_t base;
  static __device__ __forceinline__ void fetch(const Params& p, int g, int32_t len, int32_t b, int lane,
                                               int32_t& l, int32_t& ph) {
    const int32_t j = b + lane;
    l = 0;
    ph = 0;
    if (j < len) {
      l = list_at(p, g, j);
      ph = p.page_table[l];
    }
  }
  __device__ __forceinline__ void init(const Params& p, int g, int32_t len, int lane) {
    base = 0;
    fetch(p, g, len, 0, lane, l_cur, p_cur);
    fetch(p, g, len, 64, lane, l_nxt, p_nxt);
  }
  // j (wave-uniform, non-decreasing across calls) must satisfy base <= j; entries up to
  // j + 63 stay readable afterwards
  __device__ __forceinline__ void advance(const Params& p, int g, int32_t len, int32_t j, int lane) {
    if (j >= base + 64) {
      l_cur = l_nxt;
      p_cur = p_nxt;
      base += 64;
      fetch(p, g, len, base + 64, lane, l_nxt, p_nxt);
    }
  }
  __device__ __forceinline__ int32_t page(int32_t j) const {
    const int32_t k = j - base;
    const int32_t a = __builtin_amdgcn_readlane(l_cur, k & 63), b = __builtin_amdgcn_readlane(l_nxt, k & 63);
    return k < 64 ? a : b;
  }
  __device__ __forceinline__ int32_t phys(int32_t j) const {
    const int32_t k = j - base;
    const int32_t a = __builtin_amdgcn_readlane(p_cur, k & 63), b = __builtin_amdgcn_readlane(p_nxt, k & 63);
    return k < 64 ? a : b;
  }
};

// Number of leading list entries of KV head g whose logical page is <= l_max (the
// list is ascending, so the invisible entries form a suffix).  64 entries per step,
// one memory latency each.
__device__ __forceinline__ int32_t visible_len(const Params& p, int g, int64_t l_max, int lane) {
  int32_t len = list_len(p, g);
  while (len > 0) {
    const int32_t j = len - 1 - lane;
    const bool over = j >= 0 && (int64_t)list_at(p, g, j) > l_max;
    const int n_over = __builtin_popcountll(__ballot(over));
    len -= n_over;
    if (n_over < 64) break;
  }
  return len;
}

// max / sum across the two 32-lane halves of a wave (lanes l and l ^ 32).
// permlane32_swap(v, v) returns {own, partner} in lanes < 32 and {partner, own}
// in lanes >= 32, so a symmetric combine needs no select.
__device__ __forceinline__ float half_max(float v) {
  const uint32_t u = __float_as_uint(v);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float v) {
  const uint32_t u = __float_as_uint(v);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

}  // namespace oomb
