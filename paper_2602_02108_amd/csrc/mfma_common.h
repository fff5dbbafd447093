// Building blocks of the bf16 MFMA kernels (gfx950, wave64): vector types, LDS
// tile layouts and the direct global -> LDS copy helpers.  Page size 128, head dim 128.
//
// MFMA used everywhere: v_mfma_f32_32x32x16_bf16, D(32x32) += A(32x16) * B(16x32).
//   A operand: lane l holds A[l % 32][8 * (l / 32) + 0..7]
//   B operand: lane l holds B[8 * (l / 32) + 0..7][l % 32]
//   C/D:       lane l, register r holds C[8 * (r / 4) + 4 * (l / 32) + r % 4][l % 32]
//
// LDS tiles of the forward kernel (written in this byte order once per call by a layout
// kernel, "images", and copied into LDS verbatim): natural rows are 256 bytes (16 granules of
// 16 bytes), granule c of row r stored at granule position c ^ (r & 15); transposed rows are
// 128 bytes (8 granules), granule o of row d stored at o ^ ((d >> 1) & 7).  Both make the
// row-per-lane 16-byte operand reads free of bank conflicts.
//   "natural" tile:    row = token, granule c = elements 8c .. 8c+7 of the head dim.
//   "transposed" tile: row = head-dim index d; granule o = 2 * u + hh holds the
//                      eight tokens 16u + 4hh + {0,1,2,3, 8,9,10,11}; this is the
//                      token order in which a lane of C-layout half hh holds the
//                      rows of a 32x32 accumulator block, so a probability block
//                      can feed the next MFMA without any cross-lane movement.
//
// LDS tiles of the backward kernels ("row tiles"): rows in natural order, 256 bytes each, granule c
// of row r at granule position c ^ f(r), f(r) = 4 (r % 4) + (r / 4) % 4.  Such a tile serves both
// as an operand whose contraction runs along the row (16-byte row reads; 16 consecutive rows use all
// 16 positions) and as the transposed operand, fetched with ds_read_b64_tr_b16: lane i of a group of
// 16 receives word i % 4 of the 8 bytes addressed by lanes i / 4 + {0, 4, 8, 12} of its group.  With
// lane L of group gq (= lane / 16) addressing row 16 u + 8 r + 4 (gq / 2) + L / 4, columns
// 32 db + 16 (gq % 2) + 4 (L % 4) .. + 3, the lane ends up with column 32 db + lane % 32 of the rows
// 16 u + 8 r + 4 (lane / 32) + {0..3}; reads r = 0, 1 together are the eight contraction elements in
// the order of the accumulator rows (see "transposed" above).  The 32 lanes served together touch
// 4 rows x 64 bytes, which f spreads over all banks.
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

// ---- direct global -> LDS copies ----------------------------------------------------
// One wave copies `N` consecutive KiB: lane l of chunk k moves the 16 bytes at
// src + lane_off + 1024 k (lane_off = 16 l plus whatever selects the wave's share) to LDS byte
// lds_dst + 16 l + 1024 k.  src and lds_dst are wave-uniform.
//
// The loads are written in assembly on purpose: given the builtin, the compiler assumes they may
// alias any LDS read and waits for them (vmcnt(0)) before the next one, which exposes the whole
// memory latency.  A kernel that uses these copies has to order them itself: they complete in issue
// order, so "s_waitcnt vmcnt(n)" followed by a barrier publishes every copy but the n newest.  m0
// holds the LDS address of such a load; every statement names it as clobbered, so the compiler
// re-materialises whatever it keeps there itself.
template <int N>
__device__ __forceinline__ void copy_kib_to_lds(const unsigned char* src, uint32_t lane_off, uint32_t lds_dst) {
  static_assert(N == 2 || N == 4, "chunks per call");
  if (N == 2) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %2\n\t"
        "global_load_lds_dwordx4 %1, %2 offset:1024\n\t"
        :: "s"(lds_dst), "v"(lane_off), "s"(src) : "memory", "m0");
  } else {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %2\n\t"
        "global_load_lds_dwordx4 %1, %2 offset:1024\n\t"
        "global_load_lds_dwordx4 %1, %2 offset:2048\n\t"
        "global_load_lds_dwordx4 %1, %2 offset:3072\n\t"
        :: "s"(lds_dst), "v"(lane_off), "s"(src) : "memory", "m0");
  }
}
// one dword per lane (256 bytes per wave)
__device__ __forceinline__ void copy_256b_to_lds(const unsigned char* src, uint32_t lane_off, uint32_t lds_dst) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dword %1, %2\n\t"
      :: "s"(lds_dst), "v"(lane_off), "s"(src) : "memory", "m0");
}
// at most n of this wave's copies (and other vector-memory operations) are still outstanding
template <int N> __device__ __forceinline__ void wait_copies() {
  static_assert(N >= 0 && N < 16, "vmcnt");
  __builtin_amdgcn_s_waitcnt(0x0F70 | N);
}

// ---- row tiles: operand addresses and the transposing read -------------------------------
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ constexpr uint32_t row_tile_f(uint32_t r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// byte offset of granule c of row r inside a row tile
__device__ __forceinline__ constexpr uint32_t row_tile_at(uint32_t r, uint32_t c) { return r * 256 + ((c ^ row_tile_f(r)) << 4); }

// row operand of lane (lq = lane % 32, hh = lane / 32), k-step kk (dims 16 kk + 8 hh .. + 7) of a 32-row
// block: na[kk] + block offset
__device__ __forceinline__ void row_tile_addrs(int lq, int hh, uint32_t base, uint32_t (&na)[8]) {
  const uint32_t nbase = lq * 256 + ((row_tile_f(lq) ^ hh) << 4) + base;
#pragma unroll
  for (int k = 0; k < 8; ++k) na[k] = nbase ^ (k << 5);
}
// transposed operand: dim block db, rows 16 u + 8 r + ...: tt[2 db + r] + 4096 u + 2048 r + block offset
__device__ __forceinline__ void row_tile_tr_addrs(int lane, uint32_t base, uint32_t (&tt)[8]) {
  const uint32_t L = lane & 15, gq = lane >> 4;
  const uint32_t trow = 4 * (gq >> 1) + (L >> 2);
  const uint32_t tgran = (2 * (gq & 1) + ((L & 3) >> 1)) ^ (((L >> 2) << 2) | (gq >> 1));
  const uint32_t tbase = trow * 256 + (tgran << 4) + 8 * (L & 1) + base;
#pragma unroll
  for (int db = 0; db < 4; ++db) {
    tt[2 * db] = tbase ^ (db << 6);
    tt[2 * db + 1] = tbase ^ (db << 6) ^ 32;   // rows + 8: f changes by 2
  }
}
// eight 16-bit words of one column: the reads r = 0 (address a0 + off) and r = 1 (a1 + off + 2048)
__device__ __forceinline__ u32x4_t row_tile_tr_frag(const unsigned char* smem, uint32_t a0, uint32_t a1, int off) {
  const u32x2_t lo = __builtin_bit_cast(u32x2_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4_t*)(smem + (a0 + off))));
  const u32x2_t hi = __builtin_bit_cast(u32x2_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4_t*)(smem + (a1 + (off + 2048)))));
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
}

// Direct copy of 2 KiB (8 rows) of a row tile whose rows lie `row_bytes` apart in memory: the swizzle
// is applied on the source side (every lane picks the granule that belongs at its LDS position).
// off0 / off1: this lane's source offsets for the two KiB (row_tile_src_offsets); the second load
// carries an immediate of 1024 for the LDS side, which off1 compensates.
__device__ __forceinline__ void row_tile_src_offsets(int first_row, int lane, uint32_t row_bytes, uint32_t& off0, uint32_t& off1) {
  const uint32_t pos = lane & 15;
  const uint32_t r0 = first_row + (lane >> 4), r1 = r0 + 4;
  off0 = r0 * row_bytes + ((pos ^ row_tile_f(r0)) << 4);
  off1 = r1 * row_bytes + ((pos ^ row_tile_f(r1)) << 4) - 1024;
}
__device__ __forceinline__ void copy_rows_to_lds(const unsigned char* src, uint32_t off0, uint32_t off1, uint32_t lds_dst) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %3\n\t"
      "global_load_lds_dwordx4 %2, %3 offset:1024\n\t"
      :: "s"(lds_dst), "v"(off0), "v"(off1), "s"(src) : "memory", "m0");
}

// 4 KiB (16 rows): four loads, lane offsets from row_tile_src_offsets16
__device__ __forceinline__ void row_tile_src_offsets16(int lane, uint32_t row_bytes, uint32_t (&off)[4]) {
  const uint32_t pos = lane & 15;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const uint32_t r = 4 * k + (lane >> 4);   // (first row a multiple of 16: f only sees r % 16)
    off[k] = r * row_bytes + ((pos ^ row_tile_f(r)) << 4) - 1024 * k;
  }
}
__device__ __forceinline__ void copy_rows16_to_lds(const unsigned char* src, const uint32_t (&off)[4], uint32_t lds_dst) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %5\n\t"
      "global_load_lds_dwordx4 %2, %5 offset:1024\n\t"
      "global_load_lds_dwordx4 %3, %5 offset:2048\n\t"
      "global_load_lds_dwordx4 %4, %5 offset:3072\n\t"
      :: "s"(lds_dst), "v"(off[0]), "v"(off[1]), "v"(off[2]), "v"(off[3]), "s"(src) : "memory", "m0");
}

// Page list entries held in registers, 64 per window, two windows deep: lane j of a
// window holds the logical page id of list entry base + j and, in `ph`, its physical
// page -- or, with one list per query page, the position of the page in the KV head's
// union list (where its images sit).  `lid` is the list id.
// The main loops read them with v_readlane, so no iteration waits for a chain of
// dependent memory loads (selection list -> page table); the next window is
// fetched while the current one is consumed.
struct PageWindow {
  int32_t l_cur, p_cur, l_nxt, p_nxt;
  int32_t base;
  bool slots;  // (one list per query page) ph = position in the union list instead of the physical page
  __device__ __forceinline__ void fetch(const Params& p, int lid, int32_t len, int32_t b, int lane,
                                        int32_t& l, int32_t& ph) const {
    const int32_t j = b + lane;
    l = 0;
    ph = 0;
    if (j < len) {
      l = list_at(p, lid, j);
      ph = slots ? p.qp_slot[(int64_t)lid * p.sel_stride + j] : p.page_table[l];
    }
  }
  __device__ __forceinline__ void init(const Params& p, int lid, int32_t len, int lane, bool want_slots) {
    base = 0;
    slots = want_slots;
    fetch(p, lid, len, 0, lane, l_cur, p_cur);
    fetch(p, lid, len, 64, lane, l_nxt, p_nxt);
  }
  // j (wave-uniform, non-decreasing across calls) must satisfy base <= j; entries up to
  // j + 63 stay readable afterwards
  __device__ __forceinline__ void advance(const Params& p, int lid, int32_t len, int32_t j, int lane) {
    if (j >= base + 64) {
      l_cur = l_nxt;
      p_cur = p_nxt;
      base += 64;
      fetch(p, lid, len, base + 64, lane, l_nxt, p_nxt);
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

// Number of leading entries of list `lid` whose logical page is <= l_max (the
// list is ascending, so the invisible entries form a suffix).  64 entries per step,
// one memory latency each.
__device__ __forceinline__ int32_t visible_len(const Params& p, int lid, int64_t l_max, int lane) {
  int32_t len = list_len(p, lid);
  while (len > 0) {
    const int32_t j = len - 1 - lane;
    const bool over = j >= 0 && (int64_t)list_at(p, lid, j) > l_max;
    const int n_over = __builtin_popcountll(__ballot(over));
    len -= n_over;
    if (n_over < 64) break;
  }
  return len;
}

// Row tiles of the forward and dQ kernels.  Row space of a KV head: block b = tb * G + hd holds the
// 32 consecutive chunk tokens 32 tb .. 32 tb + 31 of query head g G + hd.  A tile is up to 8
// consecutive blocks, one per wave.  With one list per KV head the tiles simply partition the
// blocks; with one list per query page no tile may straddle two query pages, so every query page
// (4 G blocks) gets ceil(4 G / 8) tiles of its own and the waves beyond its last block idle along
// (they compute a copy of that block and store nothing).
struct RowTile {
  int32_t b_first, b_last;  // blocks of the tile
  uint32_t bw;              // this wave's block (clamped to b_last)
  bool valid;               // this wave owns a block
  int lid;                  // list the tile's rows use
};
__host__ __device__ __forceinline__ int32_t row_tiles_per_head(int32_t C, int32_t G, int32_t m, int qp) {
  const int32_t nblk = (C / 32) * G;
  if (!qp) return (nblk + 7) / 8;
  return m * ((nblk / m + 7) / 8);
}
__device__ __forceinline__ RowTile row_tile(const Params& p, int g, int32_t tile, int wave) {
  RowTile t;
  const int32_t nblk = (p.C / 32) * p.G;
  if (!p.qp) {
    t.b_first = tile * 8;
    t.b_last = t.b_first + 7 < nblk ? t.b_first + 7 : nblk - 1;
    t.lid = g;
  } else {
    const int32_t bpq = nblk / p.m, tpq = (bpq + 7) / 8;
    const int32_t tau = tile / tpq, sub = tile - tau * tpq;
    t.b_first = tau * bpq + sub * 8;
    t.b_last = t.b_first + 7 < (tau + 1) * bpq ? t.b_first + 7 : (tau + 1) * bpq - 1;
    t.lid = g * p.m + tau;
  }
  const int32_t b = t.b_first + wave;
  t.valid = b <= t.b_last;
  t.bw = (uint32_t)(t.valid ? b : t.b_last);
  return t;
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
