// dK / dV of the paged attention backward with bf16 MFMA (paper Sec. 3 Eq. 3 and
// Sec. 4.1: KV gradients accumulate in place in the paged gradient pool).  Page
// size 128, head dim 128.
//
// One workgroup OWNS one (KV head, selected page) -- or one slice of the query
// rows that see it -- visits those rows in blocks of 32, keeps dK^T and dV^T in
// registers and updates the page of the gradient pool once with plain loads and
// stores: no atomics, results independent of scheduling.
//
// The eight waves form four pairs, one per block of 32 keys; the two waves of a
// pair share a SIMD and split the work by role, so neither runs out of registers
// and one's matrix instructions overlap the other's vector instructions:
//   role 0 ("P"):  S = Q K^T (+ bias), P = exp2(c S), hands P to its partner through
//                  LDS, dV^T += dO^T P.      Holds the K rows and dV^T.
//   role 1 ("dS"): dP = dO V^T (+ bias), one block later dS = P o dP,
//                  dK^T += Q^T dS.           Holds the V rows and dK^T.
// In the (query x key) accumulator layout a lane owns one key column and 16 query
// rows, so the per-row statistics would differ per register.  They are folded into
// the matrix product instead: one extra MFMA adds -LSE/c (resp. -Delta) to every
// column of a row, from a per-lane (row) value split into two bf16 terms.
//
// LDS: two stages of 64 query rows x {Q natural, dO natural, Q transposed, dO
// transposed} (16 KiB each) + the P exchange (4 pairs x 2 x 2 KiB) = 144 KiB.  The
// natural tiles of both stages sit in the lower 64 KiB and the transposed tiles in
// the next 64 KiB, so that every operand address is a loop-invariant register plus
// an immediate; the loops are unrolled by two stages to make the stage a constant.
#include "mfma_common.h"

namespace oomb {

constexpr int KV_THREADS = 512;
constexpr int KV_TR = 65536;                   // first transposed tile
constexpr int KV_XCH = 131072;                 // P exchange
constexpr int KV_LDS = KV_XCH + 4 * 2 * 2048;
// tile offsets: natural Q / dO of stage st, transposed Q / dO of stage st (relative to KV_TR)
__device__ __forceinline__ constexpr int kv_nat(int st, int which) { return st * 32768 + which * 16384; }
__device__ __forceinline__ constexpr int kv_tr(int st, int which) { return st * 32768 + which * 16384; }

__device__ __forceinline__ uint4 kv_pack8(const f32x16& v, int base) {
  uint4 w;
  w.x = pack2_bf16(v[base + 0], v[base + 1]);
  w.y = pack2_bf16(v[base + 2], v[base + 3]);
  w.z = pack2_bf16(v[base + 4], v[base + 5]);
  w.w = pack2_bf16(v[base + 6], v[base + 7]);
  return w;
}

// A-operand fragment that adds `bias` (one value per row = per lane & 31) to every
// column of the row when multiplied with the "ones" B fragment: slots 0 and 1 of the
// contraction hold bias rounded to bf16 and the rounding residual.
__device__ __forceinline__ bf16x8 bias_frag(float bias, int hh) {
  const uint32_t hi = pack2_bf16(bias, 0.f) & 0xffffu;
  const uint32_t lo = pack2_bf16(bias - __uint_as_float(hi << 16), 0.f) & 0xffffu;
  uint4 w = make_uint4(hh == 0 ? (hi | (lo << 16)) : 0u, 0u, 0u, 0u);
  return as_bf16x8(w);
}

template <typename TG> __device__ __forceinline__ void kv_rmw4(TG* ptr, float a, float b, float c2, float d);
template <> __device__ __forceinline__ void kv_rmw4<float>(float* ptr, float a, float b, float c2, float d) {
  float4 v = *reinterpret_cast<float4*>(ptr);
  v.x += a; v.y += b; v.z += c2; v.w += d;
  *reinterpret_cast<float4*>(ptr) = v;
}
template <> __device__ __forceinline__ void kv_rmw4<bf16_t>(bf16_t* ptr, float a, float b, float c2, float d) {
  const uint2 v = *reinterpret_cast<uint2*>(ptr);
  uint2 w;
  w.x = pack2_bf16(__uint_as_float(v.x << 16) + a, __uint_as_float(v.x & 0xffff0000u) + b);
  w.y = pack2_bf16(__uint_as_float(v.y << 16) + c2, __uint_as_float(v.y & 0xffff0000u) + d);
  *reinterpret_cast<uint2*>(ptr) = w;
}

// Row space of a KV head: block b = tb * G + hd holds the 32 consecutive chunk tokens
// 32 tb .. 32 tb + 31 of query head g G + hd, so a 32-row MFMA block is one head and
// consecutive tokens (affine addresses, one causal offset per block).  The per-row
// statistics are laid out the same way: index 32 b + token-in-block.
//
// partial != nullptr: the unit's dK^T / dV^T go to partial[unit][2][128 keys][128 dims]
// (fp32, overwritten) instead of the pool; a second kernel adds the slices to the pool.
template <typename TG>
__global__ __launch_bounds__(KV_THREADS) void bwd_dkv_kernel(Params p, const float* __restrict__ delta_rs,
                                                             const float* __restrict__ lse2_rs, int64_t rows_pad,
                                                             int32_t max_len, int32_t n_split, int xcd_map,
                                                             float* __restrict__ partial) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, hh = lane >> 5, lq = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kbw = wave & 3, role = wave >> 2;

  // workgroup -> (KV head, list entry, row slice)
  int g;
  int32_t unit;
  if (xcd_map) {
    const int xcd = blockIdx.x & 7, per = 8 / p.Hkv;
    g = xcd % p.Hkv;
    unit = (blockIdx.x >> 3) * per + xcd / p.Hkv;
  } else {
    g = blockIdx.x % p.Hkv;
    unit = blockIdx.x / p.Hkv;
  }
  const int32_t j = unit / n_split, sp = unit % n_split;
  if (j >= max_len || j >= list_len(p, g)) return;

  const int64_t first_q = p.N - p.C;
  const int64_t l = list_at(p, g, j);
  const int64_t first = l * TP;
  const int64_t pool_off = (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride;
  const float c = p.sm_scale * 1.4426950408889634f;

  // this wave's 32 keys as B operand: K rows for role 0, V rows for role 1
  bf16x8 kvf[8];
  {
    const bf16_t* base = (role == 0 ? (const bf16_t*)p.k_pool : (const bf16_t*)p.v_pool) + pool_off +
                         (int64_t)(32 * kbw + lq) * p.pool_tok_stride;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) kvf[kk] = as_bf16x8(*reinterpret_cast<const uint4*>(base + 16 * kk + 8 * hh));
  }
  const bf16x8 ones = as_bf16x8(make_uint4(0x3f803f80u, 0u, 0u, 0u));

  // stages (2 blocks = 64 rows) this unit visits: from the first token block that can see
  // the page, cut into n_split slices
  const int32_t i_min = (int32_t)(first > first_q ? first - first_q : 0);   // first chunk token that sees the page
  const int32_t nblk_all = (p.C / 32) * p.G;
  const int32_t st_lo_all = ((i_min / 32) * p.G) >> 1, st_hi_all = nblk_all >> 1;
  const int32_t st_cnt = st_hi_all - st_lo_all;
  const int32_t s0 = st_lo_all + (int32_t)(((int64_t)st_cnt * sp) / n_split);
  const int32_t s1 = st_lo_all + (int32_t)(((int64_t)st_cnt * (sp + 1)) / n_split);
  const int32_t nb = 2 * (s1 - s0);  // blocks of 32 rows
  // offset of this lane's key behind the first chunk token; a row (chunk token i) sees the key iff i >= key_rel
  const int32_t key_rel = (int32_t)(first + 32 * kbw + lq - first_q);

  f32x16 acc[4];  // role 0: dV^T, role 1: dK^T  (128 dims x 32 keys)
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int x = 0; x < 16; ++x) acc[db][x] = 0.f;

  // LDS operand addresses: (lane base ^ constant) + immediate
  uint32_t na[8], ta[4];
  {
    const uint32_t nbase = lq * 256 + (((lq & 15) ^ hh) << 4);          // natural tiles, 16 granules per row
    const uint32_t tbase = lq * 128 + ((((lq >> 1) & 7) ^ hh) << 4);    // transposed tiles, 8 granules per row
#pragma unroll
    for (int k = 0; k < 8; ++k) na[k] = nbase ^ (k << 5);
#pragma unroll
    for (int k = 0; k < 4; ++k) ta[k] = (tbase ^ (k << 5)) + KV_TR;
  }
  const uint32_t xo = KV_XCH + kbw * 4096 + lane * 16;  // this pair's P exchange, this lane's 16 bytes

  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const uint32_t ts_bytes = (uint32_t)p.q_tok_stride * 2u;
  // Staging.  This wave moves rows 8 wave .. 8 wave + 7 of a stage's natural tiles and octet `wave`
  // (rows 16 u + 4 h2 + {0..3, 8..11}, u = wave / 2, h2 = wave % 2) of its transposed tiles; both lie
  // in block 2 s + wave / 4 of the row space.  Addresses are a wave-uniform block base plus 32-bit
  // lane offsets (kept opaque so that the loads use the scalar-base addressing form).
  uint32_t nat_off[2], tr_off[2];  // transposed: rows 16 (u & 1) + 4 h2 and + 8; + k token strides for k = 0..3
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    const uint32_t srow = 8 * wave + 4 * x + (lane >> 4);
    nat_off[x] = (srow & 31) * ts_bytes + (((lane & 15) ^ (srow & 15)) << 4);
    tr_off[x] = (uint32_t)(16 * ((wave >> 1) & 1) + 4 * (wave & 1) + 8 * x) * ts_bytes + (uint32_t)lane * 4u;
  }
  // row-space block of this wave's staging share, kept as (token block, head in group)
  int32_t ld_tb, ld_hd;
  {
    const uint32_t b = (uint32_t)(2 * s0 + (wave >> 2));
    ld_tb = (int32_t)div_g(p, b);
    ld_hd = (int32_t)b - ld_tb * p.G;
  }
  const int64_t tb_bytes = (int64_t)64 * p.q_tok_stride, hd_bytes = (int64_t)2 * p.q_head_stride;
  const int64_t g_bytes = (int64_t)g * p.G * hd_bytes;
  u32x4 qn0, qn1, don0, don1;
  uint32_t qt[8], dot[8];
  // fetch the stage whose block is (ld_tb, ld_hd), then step to the next stage (two blocks on)
  auto load_stage = [&]() __attribute__((always_inline)) {
    const int64_t bb = (int64_t)ld_tb * tb_bytes + (int64_t)ld_hd * hd_bytes + g_bytes;
    const char* qb = reinterpret_cast<const char*>(p.q) + bb;
    const char* ob = reinterpret_cast<const char*>(p.d_o) + bb;
    asm volatile("" : "+v"(nat_off[0]), "+v"(nat_off[1]), "+v"(tr_off[0]), "+v"(tr_off[1]));
    qn0 = *reinterpret_cast<const u32x4*>(qb + nat_off[0]);
    don0 = *reinterpret_cast<const u32x4*>(ob + nat_off[0]);
    qn1 = *reinterpret_cast<const u32x4*>(qb + nat_off[1]);
    don1 = *reinterpret_cast<const u32x4*>(ob + nat_off[1]);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      uint32_t oe = tr_off[e >> 2] + (uint32_t)(e & 3) * ts_bytes;
      asm volatile("" : "+v"(oe));
      qt[e] = *reinterpret_cast<const uint32_t*>(qb + oe);
      dot[e] = *reinterpret_cast<const uint32_t*>(ob + oe);
    }
    ld_hd += 2;
    if (ld_hd >= p.G) { ld_hd -= p.G; ld_tb += 1; }
    if (ld_hd >= p.G) { ld_hd -= p.G; ld_tb += 1; }
  };
  auto perm4 = [](const uint32_t* r, uint32_t sel) -> uint4 {
    uint4 w;
    w.x = __builtin_amdgcn_perm(r[1], r[0], sel);
    w.y = __builtin_amdgcn_perm(r[3], r[2], sel);
    w.z = __builtin_amdgcn_perm(r[5], r[4], sel);
    w.w = __builtin_amdgcn_perm(r[7], r[6], sel);
    return w;
  };
  const uint32_t nst_o = (8 * wave) * 256 + lane * 16;
  const uint32_t tr_o0 = KV_TR + ((2 * lane) * 8 + (wave ^ (lane & 7))) * 16, tr_o1 = tr_o0 + 128;
  auto store_stage = [&](const int st) __attribute__((always_inline)) {
    *reinterpret_cast<u32x4*>(smem + (nst_o + kv_nat(st, 0))) = qn0;
    *reinterpret_cast<u32x4*>(smem + (nst_o + kv_nat(st, 1))) = don0;
    *reinterpret_cast<u32x4*>(smem + (nst_o + (kv_nat(st, 0) + 1024))) = qn1;
    *reinterpret_cast<u32x4*>(smem + (nst_o + (kv_nat(st, 1) + 1024))) = don1;
    *reinterpret_cast<uint4*>(smem + (tr_o0 + kv_tr(st, 0))) = perm4(qt, 0x05040100u);
    *reinterpret_cast<uint4*>(smem + (tr_o1 + kv_tr(st, 0))) = perm4(qt, 0x07060302u);
    *reinterpret_cast<uint4*>(smem + (tr_o0 + kv_tr(st, 1))) = perm4(dot, 0x05040100u);
    *reinterpret_cast<uint4*>(smem + (tr_o1 + kv_tr(st, 1))) = perm4(dot, 0x07060302u);
  };

  // per-row statistic of this lane's row in block b: -LSE/c for role 0, -Delta for role 1
  const float* const stat_rs = (role == 0 ? lse2_rs : delta_rs) + (int64_t)g * rows_pad + lq;
  const float stat_scale = role == 0 ? -1.f / c : -1.f;

  // The partner's first step multiplies zeros (no previous block yet) with the transposed Q tile of
  // the second stage buffer and with the P exchange: clear both so that no stale NaN pattern is read.
  {
    const uint4 z = make_uint4(0, 0, 0, 0);
    *reinterpret_cast<uint4*>(smem + KV_TR + kv_tr(1, 0) + tid * 32) = z;
    *reinterpret_cast<uint4*>(smem + KV_TR + kv_tr(1, 0) + tid * 32 + 16) = z;
    if (role == 0) {
#pragma unroll
      for (int k = 0; k < 4; ++k) *reinterpret_cast<uint4*>(smem + (xo + k * 1024)) = z;
    }
  }
  if (nb > 0) {
    load_stage();
    store_stage(0);
  }
  __syncthreads();

  // Fragment batches: two sets of four, one batch fetched while the previous one computes.
  u32x4 fr[8];
  // natural rows of block `half` of stage st, tile `which`, k-steps 4 kq .. 4 kq + 3
  auto fetch_nat = [&](const int st, const int which, const int half, const int kq, const int set) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < 4; ++k)
      fr[set + k] = *reinterpret_cast<const u32x4*>(smem + (na[4 * kq + k] + (kv_nat(st, which) + half * 8192)));
  };
  // transposed rows (dim blocks 0..3) of key group 2 half + u of stage st, tile `which`
  auto fetch_tr = [&](const int st, const int which, const int half, const int u, const int set) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < 4; ++k)
      fr[set + k] = *reinterpret_cast<const u32x4*>(smem + (ta[2 * half + u] + (kv_tr(st, which) + k * 4096)));
  };
  auto wait4 = [&]() __attribute__((always_inline)) {
    __builtin_amdgcn_s_waitcnt(0xC47F);  // lgkmcnt(4): everything but the newest batch has arrived
    __builtin_amdgcn_sched_barrier(0);
  };
  auto frag = [&](const int idx) __attribute__((always_inline)) -> bf16x8 { return __builtin_bit_cast(bf16x8, fr[idx]); };

  // One loop iteration = one stage = two blocks, two barriers.  The next stage is fetched into
  // registers at the top and written to the other LDS buffer at the bottom.  Role 1 works one block
  // behind role 0 and finishes with one extra half step.  All code between barriers is straight-line.
  const int32_t tok_first = (int32_t)(first - first_q);
  // blocks below this index contain rows that do not see every key of the page (causal diagonal)
  const int32_t b_diag_end = tok_first + TP - 1 > 0 ? ((tok_first + TP - 1 + 31) / 32) * p.G : 0;
  if (nb > 0) {
    if (role == 0) {
      // S = Q K^T - LSE / c, P = exp2(c S) (masked), P -> partner, dV^T += dO^T P
      auto block0 = [&](const int st, const int half, const int32_t blk, const float stat_raw) __attribute__((always_inline)) {
        f32x16 sc;
        if (half == 0) fetch_nat(st, 0, 0, 0, 0);  // (block 1's first batch was fetched at the end of block 0)
        fetch_nat(st, 0, half, 1, 4);
        const bf16x8 bias = bias_frag(stat_raw * stat_scale, hh);
        wait4();
#pragma unroll
        for (int x = 0; x < 16; ++x) sc[x] = 0.f;
        sc = mfma32(bias, ones, sc);
#pragma unroll
        for (int k = 0; k < 4; ++k) sc = mfma32(frag(k), kvf[k], sc);
        __builtin_amdgcn_sched_barrier(0);
        fetch_tr(st, 1, half, 0, 0);
        wait4();
#pragma unroll
        for (int k = 0; k < 4; ++k) sc = mfma32(frag(4 + k), kvf[4 + k], sc);
        __builtin_amdgcn_sched_barrier(0);
        fetch_tr(st, 1, half, 1, 4);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int x = 0; x < 16; ++x) sc[x] = __builtin_amdgcn_exp2f(sc[x] * c);
        if (blk < b_diag_end) {  // diagonal block: rows before the key see nothing
          const int32_t rel = key_rel - 32 * (int32_t)div_g(p, (uint32_t)blk) - 4 * hh;
#pragma unroll
          for (int x = 0; x < 16; ++x)
            if (8 * (x >> 2) + (x & 3) < rel) sc[x] = 0.f;
        }
        const uint4 p0 = kv_pack8(sc, 0), p1 = kv_pack8(sc, 8);
        *reinterpret_cast<uint4*>(smem + (xo + half * 2048)) = p0;
        *reinterpret_cast<uint4*>(smem + (xo + (half * 2048 + 1024))) = p1;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int db = 0; db < 4; ++db) acc[db] = mfma32(frag(db), as_bf16x8(p0), acc[db]);
        __builtin_amdgcn_sched_barrier(0);
        if (half == 0) {
          fetch_nat(st, 0, 1, 0, 0);
          wait4();
        }
#pragma unroll
        for (int db = 0; db < 4; ++db) acc[db] = mfma32(frag(4 + db), as_bf16x8(p1), acc[db]);
        __builtin_amdgcn_sched_barrier(0);
      };
      float st_a = stat_rs[(int64_t)64 * s0], st_b = 0.f;
      auto stage0 = [&](const int32_t s, const int st) __attribute__((always_inline)) {
        const bool more = s + 1 < s1;
        if (more) load_stage();
        st_b = stat_rs[(int64_t)64 * s + 32];
        block0(st, 0, 2 * s, st_a);
        __syncthreads();
        if (more) st_a = stat_rs[(int64_t)64 * (s + 1)];
        block0(st, 1, 2 * s + 1, st_b);
        if (more) store_stage(st ^ 1);
        __syncthreads();
      };
      for (int32_t s = s0; s < s1; s += 2) {
        stage0(s, 0);
        if (s + 1 < s1) stage0(s + 1, 1);
      }
    } else {
      // dS = P o dP of the previous block (vector work first), dK^T += Q^T dS, then
      // dP = dO V^T - Delta of the current block.  The partner wave on this SIMD starts its
      // step with matrix work and does its vector work in the middle, so the two waves keep
      // both pipes busy.  dprev is consumed, dcur produced.  The previous block of half 0 is
      // block 1 of the other stage buffer.  Its first transposed batch is already in fr[0..3].
      auto step1 = [&](const int st, const int half, f32x16& dprev, f32x16& dcur, const float stat_raw) __attribute__((always_inline)) {
        const int pst = half == 0 ? st ^ 1 : st, ph = half ^ 1;
        const uint4 p0 = *reinterpret_cast<const uint4*>(smem + (xo + ph * 2048));
        const uint4 p1 = *reinterpret_cast<const uint4*>(smem + (xo + (ph * 2048 + 1024)));
        fetch_tr(pst, 0, ph, 1, 4);
        __builtin_amdgcn_s_waitcnt(0xC47F);  // lgkmcnt(4): P and the first batch have arrived
        __builtin_amdgcn_sched_barrier(0);
        const uint32_t pw[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          dprev[2 * k] *= __uint_as_float(pw[k] << 16);
          dprev[2 * k + 1] *= __uint_as_float(pw[k] & 0xffff0000u);
        }
        const uint4 s0v = kv_pack8(dprev, 0), s1v = kv_pack8(dprev, 8);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int db = 0; db < 4; ++db) acc[db] = mfma32(frag(db), as_bf16x8(s0v), acc[db]);
        __builtin_amdgcn_sched_barrier(0);
        fetch_nat(st, 1, half, 0, 0);
        wait4();
#pragma unroll
        for (int db = 0; db < 4; ++db) acc[db] = mfma32(frag(4 + db), as_bf16x8(s1v), acc[db]);
        __builtin_amdgcn_sched_barrier(0);
        fetch_nat(st, 1, half, 1, 4);
        const bf16x8 bias = bias_frag(stat_raw * stat_scale, hh);
        wait4();
#pragma unroll
        for (int x = 0; x < 16; ++x) dcur[x] = 0.f;
        dcur = mfma32(bias, ones, dcur);
#pragma unroll
        for (int k = 0; k < 4; ++k) dcur = mfma32(frag(k), kvf[k], dcur);
        __builtin_amdgcn_sched_barrier(0);
        fetch_tr(st, 0, half, 0, 0);  // first transposed batch of the next step (this block becomes its previous one)
        wait4();
#pragma unroll
        for (int k = 0; k < 4; ++k) dcur = mfma32(frag(4 + k), kvf[4 + k], dcur);
        __builtin_amdgcn_sched_barrier(0);
      };
      f32x16 dpa, dpb;  // dP of even / odd blocks
#pragma unroll
      for (int x = 0; x < 16; ++x) dpb[x] = 0.f;
      float st_a = stat_rs[(int64_t)64 * s0], st_b = 0.f;
      fetch_tr(1, 0, 1, 0, 0);  // zeros (cleared above): first batch of the first step
      auto stage1 = [&](const int32_t s, const int st) __attribute__((always_inline)) {
        const bool more = s + 1 < s1;
        if (more) load_stage();
        st_b = stat_rs[(int64_t)64 * s + 32];
        step1(st, 0, dpb, dpa, st_a);
        __syncthreads();
        if (more) st_a = stat_rs[(int64_t)64 * (s + 1)];
        step1(st, 1, dpa, dpb, st_b);
        if (more) store_stage(st ^ 1);
        __syncthreads();
      };
      int32_t s = s0;
      for (; s < s1; s += 2) {
        stage1(s, 0);
        if (s + 1 < s1) stage1(s + 1, 1);
      }
      // the last block's dS and dK^T contribution: its stage buffer is ((s1 - s0 - 1) & 1)
      {
        const uint4 p0 = *reinterpret_cast<const uint4*>(smem + (xo + 2048));
        const uint4 p1 = *reinterpret_cast<const uint4*>(smem + (xo + (2048 + 1024)));
        const uint32_t pw[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          dpb[2 * k] *= __uint_as_float(pw[k] << 16);
          dpb[2 * k + 1] *= __uint_as_float(pw[k] & 0xffff0000u);
        }
        const uint4 s0v = kv_pack8(dpb, 0), s1v = kv_pack8(dpb, 8);
        if (((s1 - s0 - 1) & 1) == 0) fetch_tr(0, 0, 1, 1, 4); else fetch_tr(1, 0, 1, 1, 4);
#pragma unroll
        for (int db = 0; db < 4; ++db) acc[db] = mfma32(frag(db), as_bf16x8(s0v), acc[db]);
#pragma unroll
        for (int db = 0; db < 4; ++db) acc[db] = mfma32(frag(4 + db), as_bf16x8(s1v), acc[db]);
      }
    }
  }

  // epilogue: role 0 holds dV^T, role 1 holds dK^T (to be scaled), lane = key, 4 consecutive dims per group
  const float scale = role == 0 ? 1.f : p.sm_scale;
  if (partial) {
    float* dst = partial + ((((int64_t)g * max_len + j) * n_split + sp) * 2 + (role == 0 ? 1 : 0)) * (TP * HD) +
                 (int64_t)(32 * kbw + lq) * HD;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        float4 v = {acc[db][4 * a + 0] * scale, acc[db][4 * a + 1] * scale, acc[db][4 * a + 2] * scale,
                    acc[db][4 * a + 3] * scale};
        *reinterpret_cast<float4*>(dst + 32 * db + 8 * a + 4 * hh) = v;
      }
  } else {
    TG* pool = (TG*)(role == 0 ? p.dv_pool : p.dk_pool) + pool_off + (int64_t)(32 * kbw + lq) * p.pool_tok_stride;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a)
        kv_rmw4<TG>(pool + 32 * db + 8 * a + 4 * hh, acc[db][4 * a + 0] * scale, acc[db][4 * a + 1] * scale,
                    acc[db][4 * a + 2] * scale, acc[db][4 * a + 3] * scale);
  }
}

// pool page += sum over the n_split slices of partial (one thread per 4 dims)
template <typename TG>
__global__ __launch_bounds__(256) void bwd_dkv_reduce_kernel(Params p, const float* __restrict__ partial,
                                                             int32_t max_len, int32_t n_split) {
  const int g = blockIdx.z;
  const int32_t j = blockIdx.y;
  if (j >= list_len(p, g)) return;
  const int which = blockIdx.x >> 4;                       // 0: dK, 1: dV
  const int e4 = ((blockIdx.x & 15) * 256 + threadIdx.x);  // float4 index inside the 128 x 128 page
  const int key = e4 >> 5, d4 = (e4 & 31) * 4;
  const int64_t l = list_at(p, g, j);
  const int64_t pool_off = (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride +
                           (int64_t)key * p.pool_tok_stride + d4;
  float4 s = {0.f, 0.f, 0.f, 0.f};
  for (int sp = 0; sp < n_split; ++sp) {
    const float4 v = *reinterpret_cast<const float4*>(
        partial + ((((int64_t)g * max_len + j) * n_split + sp) * 2 + which) * (TP * HD) + key * HD + d4);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  TG* pool = (TG*)(which == 0 ? p.dk_pool : p.dv_pool) + pool_off;
  kv_rmw4<TG>(pool, s.x, s.y, s.z, s.w);
}

size_t dkv_partial_bytes(const Params& p, int32_t max_len, int32_t n_split) {
  if (n_split <= 1) return 0;
  return (size_t)p.Hkv * (size_t)max_len * (size_t)n_split * 2 * TP * HD * sizeof(float);
}

// Slices per page: enough units (about 8 rounds of 256 workgroups) for the tail of the last
// round to be short, without making the second-stage reduction large.
int32_t dkv_splits(const Params& p, int32_t max_len) {
  const int64_t units = (int64_t)p.Hkv * max_len;
  if (units <= 0) return 1;
  const int64_t want = (2048 + units - 1) / units;
  return (int32_t)(want < 1 ? 1 : (want > 4 ? 4 : want));
}

hipError_t launch_bwd_dkv_mfma(const Params& p, const float* delta_rs, const float* lse2_rs, int64_t rows_pad,
                               int32_t max_len, float* partial_ws, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)bwd_dkv_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, KV_LDS);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void*)bwd_dkv_kernel<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, KV_LDS);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int32_t n_split = dkv_splits(p, max_len);
  float* partial = n_split > 1 ? partial_ws : nullptr;
  const int xcd_map = (p.Hkv <= 8 && 8 % p.Hkv == 0) ? 1 : 0;
  const int per = xcd_map ? 8 / p.Hkv : 1;
  const int64_t units = (int64_t)max_len * n_split;
  const unsigned blocks = xcd_map ? 8u * (unsigned)((units + per - 1) / per) : (unsigned)units * p.Hkv;
  {
    ProfScope prof_("bwd_dkv_mfma", st);
    if (p.grad_is_bf16)
      bwd_dkv_kernel<bf16_t><<<dim3(blocks), dim3(KV_THREADS), KV_LDS, st>>>(p, delta_rs, lse2_rs, rows_pad, max_len,
                                                                              n_split, xcd_map, partial);
    else
      bwd_dkv_kernel<float><<<dim3(blocks), dim3(KV_THREADS), KV_LDS, st>>>(p, delta_rs, lse2_rs, rows_pad, max_len,
                                                                             n_split, xcd_map, partial);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (n_split > 1) {
    ProfScope prof_("bwd_dkv_reduce", st);
    dim3 grid(32, (unsigned)max_len, (unsigned)p.Hkv);
    if (p.grad_is_bf16) bwd_dkv_reduce_kernel<bf16_t><<<grid, dim3(256), 0, st>>>(p, partial, max_len, n_split);
    else bwd_dkv_reduce_kernel<float><<<grid, dim3(256), 0, st>>>(p, partial, max_len, n_split);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace oomb
