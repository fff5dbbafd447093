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
// rows, so the per-row statistics differ per register.  They are folded into the matrix
// product: the accumulator chain of a block does not start from zero but from -LSE/c
// (resp. -Delta) of the register's row, read from the stage's bias words (fp32, prepared
// once per call by the kernel that computes Delta) straight into the accumulator registers.
//
// LDS: four stage buffers of 64 query rows x {Q, dO} (16 KiB each, rows in natural order) + the
// P exchange (4 pairs x 2 x 2 KiB) + bias words = 146 KiB.  Both products of a role read the same
// tiles: the chain takes whole rows (16-byte reads), the transposed-tile product takes its
// operand with the transposing LDS read of gfx950 (ds_read_b64_tr_b16: 16 lanes hand in 16 rows
// of four 16-bit words and get back four rows of one column each), so no transposed copy of Q / dO
// exists anywhere.  The Q tiles of all buffers sit in the lower 64 KiB and the dO tiles in the
// next 64 KiB, so that every operand address is a loop-invariant register plus an immediate below
// 64 KiB; the loops are unrolled by four stages to make the buffer a constant.
#include "mfma_common.h"
#include "launch.h"

namespace oomb {

constexpr int KV_THREADS = 512;
constexpr int KV_BUFS = 4;                     // stage buffers
constexpr int KV_DO = 65536;                   // first dO tile (the Q tiles start at 0)
constexpr int KV_XCH = 131072;                 // P exchange
constexpr int KV_BIAS = KV_XCH + 4 * 2 * 2048;  // bias words: [stage buffer][role][64 rows]
constexpr int KV_LDS = KV_BIAS + KV_BUFS * 512;
// offset of block `half` of stage buffer st inside the Q tiles or the dO tiles
__device__ __forceinline__ constexpr int kv_blk(int st, int half) { return st * 16384 + half * 8192; }

__device__ __forceinline__ uint4 kv_pack8(const f32x16& v, int base) {
  uint4 w;
  w.x = pack2_bf16(v[base + 0], v[base + 1]);
  w.y = pack2_bf16(v[base + 2], v[base + 3]);
  w.z = pack2_bf16(v[base + 4], v[base + 5]);
  w.w = pack2_bf16(v[base + 6], v[base + 7]);
  return w;
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
__global__ __launch_bounds__(KV_THREADS) void bwd_dkv_kernel(Params p, const float* __restrict__ bias,
                                                             int32_t n_stages, int32_t max_len, int32_t n_split,
                                                             int xcd_map, float* __restrict__ partial) {
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
  // one list per KV head: unit = (list entry, one of n_split equal slices of the rows that see it).
  // one list per query page: unit = entry of the work table built with the inverse lists: a page of
  // the union list and up to 8 of the query pages whose list holds it.
  int32_t j, sp = 0, q0 = 0, qc = 0, pslot = -1;
  if (p.qp) {
    const int32_t n_units = p.unit_count[g];
    if (unit >= n_units) return;
    // (the table is in ascending page order; the chunk's own pages, seen by the most rows, come last: start them first)
    const int4 un = p.units[(int64_t)g * p.max_units + (n_units - 1 - unit)];
    j = un.x; q0 = un.y; qc = un.z; pslot = un.w;
  } else {
    j = unit / n_split;
    sp = unit % n_split;
    if (j >= max_len || j >= list_len(p, g)) return;
  }

  const int64_t first_q = p.N - p.C;
  const int64_t l = owned_at(p, g, j);
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

  // stages (2 blocks = 64 rows) this unit visits: from the first token block that can see
  // the page, cut into n_split slices
  const int32_t i_min = (int32_t)(first > first_q ? first - first_q : 0);   // first chunk token that sees the page
  const int32_t nblk_all = (p.C / 32) * p.G;
  const int32_t st_lo_all = ((i_min / 32) * p.G) >> 1, st_hi_all = nblk_all >> 1;
  const int32_t st_cnt = st_hi_all - st_lo_all;
  // stage counter range [s0, s1).  One list per KV head: the stages themselves.  One list per query
  // page: stage v of the unit is stage v % spq of query page tau[v / spq] (spq stages per query page)
  const int32_t spq = (p.P / 32) * p.G / 2;
  const int32_t s0 = p.qp ? 0 : st_lo_all + (int32_t)(((int64_t)st_cnt * sp) / n_split);
  const int32_t s1 = p.qp ? qc * spq : st_lo_all + (int32_t)(((int64_t)st_cnt * (sp + 1)) / n_split);
  const int32_t nb = 2 * (s1 - s0);  // blocks of 32 rows
  int32_t tau_v = 0;                 // lane k: k-th query page of this unit
  if (p.qp && lane < qc)
    tau_v = p.inv_qp[(int64_t)g * p.m * p.sel_stride + p.inv_off[(int64_t)g * (p.un_stride + 1) + j] + q0 + lane];
  // walking the stages in order: real stage index of the current counter value and of the next one
  int32_t walk_q = 0, walk_r = 0;
  auto real_first = [&]() __attribute__((always_inline)) -> int32_t {
    return p.qp ? __builtin_amdgcn_readlane(tau_v, 0) * spq : s0;
  };
  auto real_next = [&](const int32_t cur) __attribute__((always_inline)) -> int32_t {
    if (!p.qp) return cur + 1;
    if (++walk_r == spq) {
      walk_r = 0;
      ++walk_q;
    }
    return __builtin_amdgcn_readlane(tau_v, walk_q & 63) * spq + walk_r;  // (past the unit's end: unused)
  };
  // offset of this lane's key behind the first chunk token; a row (chunk token i) sees the key iff i >= key_rel
  const int32_t key_rel = (int32_t)(first + 32 * kbw + lq - first_q);

  f32x16 acc[4];  // role 0: dV^T, role 1: dK^T  (128 dims x 32 keys)
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int x = 0; x < 16; ++x) acc[db][x] = 0.f;

  // LDS operand addresses: (lane base ^ constant) + immediate.  Role 0 chains on Q rows and takes
  // dO^T for its transposed-tile product, role 1 chains on dO rows and takes Q^T.
  uint32_t na[8], tt[8];
  row_tile_addrs(lq, hh, role == 0 ? 0 : KV_DO, na);
  row_tile_tr_addrs(lane, role == 0 ? KV_DO : 0, tt);
  const uint32_t xo = KV_XCH + kbw * 4096 + lane * 16;  // this pair's P exchange, this lane's 16 bytes

  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  // Staging.  The query-side tiles of a stage are 2 x 32 rows of Q and of dO, each row 256 contiguous
  // bytes of the chunk's tensors; they are copied with direct global -> LDS loads (no staging
  // registers, so several stages of copies can be in flight; the swizzle is applied on the source
  // side): every wave moves 16 rows (4 KiB) -- waves 0..3 those of Q, 4..7 those of dO -- and waves
  // 0 and 1 also the stage's bias words.  This kernel orders the copies itself: they complete in
  // issue order, so "at most n outstanding" before a barrier publishes everything older than the
  // newest n.
  uint32_t cp_rows[4];
  row_tile_src_offsets16(lane, (uint32_t)(p.q_tok_stride * 2), cp_rows);
  const unsigned char* cp_src = (const unsigned char*)(wave < 4 ? p.q : p.d_o);
  const float* bias_g = bias + (int64_t)g * n_stages * 128;
  const uint32_t cp_bias = 256 * wave + 4 * lane;   // (waves 0, 1) lane offset inside the bias words
  const uint32_t cp_dst = (wave >> 2) * KV_DO + (wave & 3) * 4096;
  // stage s -> stage buffer st.  The buffer's last readers must have passed a barrier.
  auto copy_stage = [&](const int32_t s, const int st) __attribute__((always_inline)) {
    const uint32_t blk = (uint32_t)(2 * s + ((wave & 3) >> 1)), tb = div_g(p, blk);   // this wave's block: one head, 32 tokens
    const int64_t row0 = (int64_t)(32 * tb + 16 * (wave & 1)) * p.q_tok_stride +
                         (int64_t)(g * p.G + (int)(blk - tb * p.G)) * p.q_head_stride;
    copy_rows16_to_lds(cp_src + row0 * 2, cp_rows, st * 16384 + cp_dst);
    if (wave < 2) copy_256b_to_lds((const unsigned char*)(bias_g + (int64_t)s * 128), cp_bias, KV_BIAS + st * 512 + 256 * wave);
  };
  // all but the newest n stages of copies have landed (a stage is 4 loads, 5 for waves 0 and 1)
  auto wait_stages = [&](const int n) __attribute__((always_inline)) {
    if (n >= 2) {
      if (wave < 2) wait_copies<10>();
      else wait_copies<8>();
    } else if (n == 1) {
      if (wave < 2) wait_copies<5>();
      else wait_copies<4>();
    } else {
      wait_copies<0>();
    }
  };
  // this role's bias words of block `half` of stage buffer st, as the initial value of a (query x key)
  // accumulator: register x belongs to row 8 (x / 4) + 4 hh + x % 4 of the block
  const uint32_t bias_o = KV_BIAS + (role * 64 + 4 * hh) * 4;
  auto load_bias = [&](const int st, const int half, f32x16& chain) __attribute__((always_inline)) {
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const float4 v = *reinterpret_cast<const float4*>(smem + (bias_o + (st * 512 + half * 128 + a * 32)));
      chain[4 * a + 0] = v.x; chain[4 * a + 1] = v.y; chain[4 * a + 2] = v.z; chain[4 * a + 3] = v.w;
    }
  };

  // Both roles multiply the transposed tile of the previous block one step late; in the very first
  // step that "previous block" is zeros times block 1 of the last stage buffer.  Clear those
  // blocks and the P exchange so that no stale NaN pattern is read.
  {
    const uint4 z = make_uint4(0, 0, 0, 0);
    unsigned char* blk = smem + ((tid >> 8) * KV_DO + kv_blk(KV_BUFS - 1, 1) + (tid & 255) * 32);
    *reinterpret_cast<uint4*>(blk) = z;
    *reinterpret_cast<uint4*>(blk + 16) = z;
    if (role == 0) {
#pragma unroll
      for (int k = 0; k < 4; ++k) *reinterpret_cast<uint4*>(smem + (xo + k * 1024)) = z;
    }
  }
  // real stages of the stage being computed and of the two after it (their copies are under way)
  int32_t rs = real_first(), rs1 = real_next(rs), rs2 = real_next(rs1);
  const int32_t n_st = s1 - s0;
  // (every load issued so far -- the K / V rows -- is waited for here, once, so that no wait for
  // them is left inside the loops, where it would drain the copies under way)
  wait_copies<0>();
  if (n_st > 0) copy_stage(rs, 0);
  if (n_st > 1) copy_stage(rs1, 1);
  if (n_st > 2) copy_stage(rs2, 2);
  wait_stages(n_st > 2 ? 2 : n_st - 1);
  __syncthreads();

  // The matrix phase of a step, the same for both roles: the accumulator chain of the current block
  // (S = bias + Q K^T for role 0, dP = bias + dO V^T for role 1: A = rows of the role's chain tile,
  // B = this wave's K or V rows) interleaved with the transposed-tile product of the PREVIOUS block
  // (dV^T += dO^T P resp. dK^T += Q^T dS: A = transposed reads of the role's other tile, B = b0 / b1),
  // so that neighbouring matrix instructions never depend on each other.  Batch j of four: k-steps
  // 2j, 2j+1 of the chain, dim blocks 2 (j % 2), + 1 of key group j / 2.  One batch is fetched ahead;
  // one wait per batch.  The previous block of half 0 is block 1 of the previous stage buffer.
  u32x4 fr[12];
  auto fetch = [&](const int st, const int half, const int j, const int set) __attribute__((always_inline)) {
    const int pst = half == 0 ? (st + KV_BUFS - 1) % KV_BUFS : st, ph = half ^ 1, u = j >> 1, db = 2 * (j & 1);
    const int po = kv_blk(pst, ph) + u * 4096;
    fr[set + 0] = *reinterpret_cast<const u32x4*>(smem + (na[2 * j] + kv_blk(st, half)));
    fr[set + 1] = row_tile_tr_frag(smem, tt[2 * db], tt[2 * db + 1], po);
    fr[set + 2] = *reinterpret_cast<const u32x4*>(smem + (na[2 * j + 1] + kv_blk(st, half)));
    fr[set + 3] = row_tile_tr_frag(smem, tt[2 * db + 2], tt[2 * db + 3], po);
  };
  auto frag = [&](const int idx) __attribute__((always_inline)) -> bf16x8 { return __builtin_bit_cast(bf16x8, fr[idx]); };
  // batches 0 and 1 must already be on their way into fr[0..3] and fr[4..7]; three sets rotate, two
  // batches (six LDS reads each) are in flight while one computes
  // `chain` enters holding the bias words of its rows (load_bias, issued before the fragment fetches)
  auto matrix_phase = [&](const int st, const int half, f32x16& chain, const uint4& b0, const uint4& b1)
      __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int set = 4 * (j % 3), db = 2 * (j & 1);
      if (j < 2) {
        fetch(st, half, j + 2, 4 * ((j + 2) % 3));
        __builtin_amdgcn_s_waitcnt(0xCC7F);  // lgkmcnt(12): this batch has arrived
      } else if (j == 2) {
        __builtin_amdgcn_s_waitcnt(0xC67F);  // lgkmcnt(6)
      } else {
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
      }
      __builtin_amdgcn_sched_barrier(0);
      const bf16x8 bb = as_bf16x8(j < 2 ? b0 : b1);
      chain = mfma32(frag(set + 0), kvf[2 * j], chain);
      acc[db] = mfma32(frag(set + 1), bb, acc[db]);
      chain = mfma32(frag(set + 2), kvf[2 * j + 1], chain);
      acc[db + 1] = mfma32(frag(set + 3), bb, acc[db + 1]);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // the transposed-tile product of the last block (it has no following step): 8 matrix instructions
  auto flush_phase = [&](const uint4& b0, const uint4& b1) __attribute__((always_inline)) {
    const uint32_t last = (uint32_t)((n_st - 1) & (KV_BUFS - 1)) * 16384 + 8192;  // block 1 of the last stage's buffer
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
      for (int k = 0; k < 4; ++k) fr[k] = row_tile_tr_frag(smem, tt[2 * k] + last, tt[2 * k + 1] + last, u * 4096);
#pragma unroll
      for (int k = 0; k < 4; ++k) acc[k] = mfma32(frag(k), as_bf16x8(u == 0 ? b0 : b1), acc[k]);
    }
  };

  // One call = one stage = two blocks, two barriers.  After the first barrier every wave has finished
  // the previous stage's last block, so that stage's buffer takes the copy of the stage three ahead;
  // before the second barrier the next stage must have landed (the copies of the two stages after it
  // may still be in flight).  Role 0's matrix phase comes first in a step and its vector phase last;
  // role 1 is the other way round, so the two waves of a SIMD keep both pipes busy.  Role 1 works one
  // block behind role 0 (it needs the P of the block), and both add the transposed-tile product one
  // step late.
  auto stage_sync = [&](const int32_t s, const int st, auto&& second_step) __attribute__((always_inline)) {
    __syncthreads();
    const int32_t rs3 = real_next(rs2);
    if (s + 3 < s1) copy_stage(rs3, (st + 3) % KV_BUFS);
    second_step();
    wait_stages((s + 2 < s1 ? 1 : 0) + (s + 3 < s1 ? 1 : 0));
    __syncthreads();
    rs = rs1; rs1 = rs2; rs2 = rs3;
  };
  const int32_t tok_first = (int32_t)(first - first_q);
  // blocks below this index contain rows that do not see every key of the page (causal diagonal)
  const int32_t b_diag_end = tok_first + TP - 1 > 0 ? ((tok_first + TP - 1 + 31) / 32) * p.G : 0;
  if (nb > 0) {
    if (role == 0) {
      // matrix: S = Q K^T - LSE / c  ||  dV^T += dO^T P(previous block);  vector: P = exp2(c S), masked, -> partner
      uint4 p0 = make_uint4(0, 0, 0, 0), p1 = p0;
      auto step0 = [&](const int st, const int half, const int32_t blk) __attribute__((always_inline)) {
        f32x16 sc;
        load_bias(st, half, sc);
        fetch(st, half, 0, 0);
        fetch(st, half, 1, 4);
        matrix_phase(st, half, sc, p0, p1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int x = 0; x < 16; ++x) sc[x] = __builtin_amdgcn_exp2f(sc[x] * c);
        if (blk < b_diag_end) {  // diagonal block: rows before the key see nothing
          const int32_t rel = key_rel - 32 * (int32_t)div_g(p, (uint32_t)blk) - 4 * hh;
#pragma unroll
          for (int x = 0; x < 16; ++x)
            if (8 * (x >> 2) + (x & 3) < rel) sc[x] = 0.f;
        }
        p0 = kv_pack8(sc, 0);
        p1 = kv_pack8(sc, 8);
        *reinterpret_cast<uint4*>(smem + (xo + half * 2048)) = p0;
        *reinterpret_cast<uint4*>(smem + (xo + (half * 2048 + 1024))) = p1;
      };
      // s: stage counter; rs: its real stage
      auto stage0 = [&](const int32_t s, const int st) __attribute__((always_inline)) {
        const int32_t blk = 2 * rs;
        step0(st, 0, blk);
        stage_sync(s, st, [&]() __attribute__((always_inline)) { step0(st, 1, blk + 1); });
      };
      for (int32_t s = s0; s < s1; s += 4) {
        stage0(s, 0);
        if (s + 1 < s1) stage0(s + 1, 1);
        if (s + 2 < s1) stage0(s + 2, 2);
        if (s + 3 < s1) stage0(s + 3, 3);
      }
      flush_phase(p0, p1);
    } else {
      // vector: dS = P o dP of the previous block;  matrix: dP = dO V^T - Delta  ||  dK^T += Q^T dS(previous block)
      auto step1 = [&](const int st, const int half, f32x16& dprev, f32x16& dcur) __attribute__((always_inline)) {
        const int ph = half ^ 1;
        load_bias(st, half, dcur);
        const uint4 p0 = *reinterpret_cast<const uint4*>(smem + (xo + ph * 2048));
        const uint4 p1 = *reinterpret_cast<const uint4*>(smem + (xo + (ph * 2048 + 1024)));
        fetch(st, half, 0, 0);
        fetch(st, half, 1, 4);
        __builtin_amdgcn_s_waitcnt(0xCC7F);  // lgkmcnt(12): P has arrived
        __builtin_amdgcn_sched_barrier(0);
        const uint32_t pw[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          dprev[2 * k] *= __uint_as_float(pw[k] << 16);
          dprev[2 * k + 1] *= __uint_as_float(pw[k] & 0xffff0000u);
        }
        const uint4 s0v = kv_pack8(dprev, 0), s1v = kv_pack8(dprev, 8);
        __builtin_amdgcn_sched_barrier(0);
        matrix_phase(st, half, dcur, s0v, s1v);
      };
      f32x16 dpa, dpb;  // dP of even / odd blocks
#pragma unroll
      for (int x = 0; x < 16; ++x) dpb[x] = 0.f;
      auto stage1 = [&](const int32_t s, const int st) __attribute__((always_inline)) {
        step1(st, 0, dpb, dpa);
        stage_sync(s, st, [&]() __attribute__((always_inline)) { step1(st, 1, dpa, dpb); });
      };
      for (int32_t s = s0; s < s1; s += 4) {
        stage1(s, 0);
        if (s + 1 < s1) stage1(s + 1, 1);
        if (s + 2 < s1) stage1(s + 2, 2);
        if (s + 3 < s1) stage1(s + 3, 3);
      }
      // the last block's dS and dK^T contribution
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
        flush_phase(s0v, s1v);
      }
    }
  }

  // epilogue: role 0 holds dV^T, role 1 holds dK^T (to be scaled), lane = key, 4 consecutive dims per group
  const float scale = role == 0 ? 1.f : p.sm_scale;
  // slices of a page go to fp32 partial pages (added to the pool by the reduce kernel), whole pages
  // straight into the pool
  const int64_t part_idx = p.qp ? (int64_t)pslot : (partial ? ((int64_t)g * max_len + j) * n_split + sp : -1);
  if (part_idx >= 0) {
    float* dst = partial + (part_idx * 2 + (role == 0 ? 1 : 0)) * (TP * HD) + (int64_t)(32 * kbw + lq) * HD;
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
  int32_t j = blockIdx.y;
  int64_t first_part;
  if (p.qp) {  // only the pages that were cut into several units have partial pages: blockIdx.y walks their list
    if (j >= p.multi_count[g]) return;
    j = p.multi_list[(int64_t)g * p.max_multi + j];
    n_split = p.un_ns[(int64_t)g * p.un_stride + j];
    first_part = p.un_pbase[(int64_t)g * p.un_stride + j];
  } else {
    if (j >= list_len(p, g)) return;
    first_part = ((int64_t)g * max_len + j) * n_split;
  }
  const int which = blockIdx.x >> 4;                       // 0: dK, 1: dV
  const int e4 = ((blockIdx.x & 15) * 256 + threadIdx.x);  // float4 index inside the 128 x 128 page
  const int key = e4 >> 5, d4 = (e4 & 31) * 4;
  const int64_t l = owned_at(p, g, j);
  const int64_t pool_off = (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride +
                           (int64_t)key * p.pool_tok_stride + d4;
  float4 s = {0.f, 0.f, 0.f, 0.f};
  for (int sp = 0; sp < n_split; ++sp) {
    // (read once: non-temporal, so that the partial pages do not push anything else out of the caches)
    typedef float f32x4_t __attribute__((ext_vector_type(4)));
    const f32x4_t v = __builtin_nontemporal_load(
        reinterpret_cast<const f32x4_t*>(partial + ((first_part + sp) * 2 + which) * (TP * HD) + key * HD + d4));
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  TG* pool = (TG*)(which == 0 ? p.dk_pool : p.dv_pool) + pool_off;
  kv_rmw4<TG>(pool, s.x, s.y, s.z, s.w);
}

size_t dkv_partial_bytes(const Params& p, int32_t max_len, int32_t n_split) {
  if (p.qp) return (size_t)p.Hkv * (size_t)qp_max_pslots(p, p.sel_stride) * 2 * TP * HD * sizeof(float);
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

hipError_t launch_bwd_dkv_mfma(const Params& p, const float* bias, int32_t n_stages, int32_t max_len,
                               float* partial_ws, hipStream_t st) {
  static DeviceOnce lds_once_f32, lds_once_bf16;
  if (hipError_t e = ensure_max_dynamic_lds(lds_once_f32, (const void*)bwd_dkv_kernel<float>, KV_LDS); e != hipSuccess) return e;
  if (hipError_t e = ensure_max_dynamic_lds(lds_once_bf16, (const void*)bwd_dkv_kernel<bf16_t>, KV_LDS); e != hipSuccess) return e;
  // (one list per query page: the units come from the device-built table; the grid covers its capacity)
  const int32_t n_split = p.qp ? 1 : dkv_splits(p, max_len);
  float* partial = (p.qp || n_split > 1) ? partial_ws : nullptr;
  const int xcd_map = (p.Hkv <= 8 && 8 % p.Hkv == 0) ? 1 : 0;
  const int per = xcd_map ? 8 / p.Hkv : 1;
  const int64_t units = p.qp ? (int64_t)p.max_units : (int64_t)max_len * n_split;
  const unsigned blocks = xcd_map ? 8u * (unsigned)((units + per - 1) / per) : (unsigned)units * p.Hkv;
  {
    ProfScope prof_("bwd_dkv_mfma", st);
    if (p.grad_is_bf16)
      bwd_dkv_kernel<bf16_t><<<dim3(blocks), dim3(KV_THREADS), KV_LDS, st>>>(p, bias, n_stages, max_len, n_split, xcd_map,
                                                                              partial);
    else
      bwd_dkv_kernel<float><<<dim3(blocks), dim3(KV_THREADS), KV_LDS, st>>>(p, bias, n_stages, max_len, n_split, xcd_map,
                                                                             partial);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (p.qp || n_split > 1) {
    ProfScope prof_("bwd_dkv_reduce", st);
    dim3 grid(32, (unsigned)(p.qp ? p.max_multi : max_len), (unsigned)p.Hkv);
    if (p.grad_is_bf16) bwd_dkv_reduce_kernel<bf16_t><<<grid, dim3(256), 0, st>>>(p, partial, max_len, n_split);
    else bwd_dkv_reduce_kernel<float><<<grid, dim3(256), 0, st>>>(p, partial, max_len, n_split);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace oomb
