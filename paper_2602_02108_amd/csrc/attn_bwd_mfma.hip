// Paged attention backward with bf16 MFMA (paper Sec. 3 Eq. 3 and Sec. 4.1: dK/dV
// are accumulated in place into the paged gradient pool; Sec. 4.2: the forward's
// page list is reused).  Page size 128, head dim 128.
//
// Kernels:
//   bwd_prep   : Delta = <dO, O> and LSE * log2(e), both re-laid out in the KV head's
//                "row space" r = 32 b + token-in-block (block b = tb * G + head in group)
//                and padded to whole tiles; and the bias words of the dK/dV kernel: per
//                64-row stage float [which][row], -LSE / c for which = 0 and -Delta for
//                which = 1, from which that kernel starts its accumulator chains.
//   bwd_dq     : parallel over 256-row tiles (like the forward); per 32-key block:
//                S^T = K Q^T, dP^T = V dO^T, dS^T = P^T o (dP^T - Delta),
//                dQ^T += K^T dS^T.  Every lane owns one query row.  K and V half tiles come
//                straight from the paged pools.
//   bwd_dkv    : (attn_bwd_dkv_mfma.hip) one workgroup OWNS one (KV head, selected page).
#include "mfma_common.h"
#include "launch.h"

namespace oomb {

constexpr int BW_WAVES = 8;
constexpr int BW_THREADS = BW_WAVES * 64;
constexpr int DQ_ROWS = 256;
constexpr int ROW_PAD = 256;  // row-space statistics are padded to a multiple of this

__device__ __forceinline__ uint4 pack8(const f32x16& v, int base) {
  uint4 w;
  w.x = pack2_bf16(v[base + 0], v[base + 1]);
  w.y = pack2_bf16(v[base + 2], v[base + 3]);
  w.z = pack2_bf16(v[base + 4], v[base + 5]);
  w.w = pack2_bf16(v[base + 6], v[base + 7]);
  return w;
}

static inline int64_t rows_padded(const Params& p) {
  const int64_t rows = (int64_t)p.C * p.G;
  return (rows + ROW_PAD - 1) / ROW_PAD * ROW_PAD;
}

// ---------------------------------------------------------------------------------
// 16 lanes per row (8 elements each), 4 rows per wave.
__global__ __launch_bounds__(256) void bwd_prep_kernel(Params p, float* __restrict__ delta_rs,
                                                       float* __restrict__ lse2_rs, int64_t rows_pad,
                                                       float* __restrict__ bias, int32_t n_stages) {
  const int lane16 = threadIdx.x & 15;
  const int64_t idx = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);  // over Hkv * rows_pad
  if (idx >= (int64_t)p.Hkv * rows_pad) return;
  const int g = (int)(idx / rows_pad);
  const int64_t r = idx % rows_pad;
  const int64_t rows_total = (int64_t)p.C * p.G;
  float acc = 0.f, l2 = 1e30f;
  if (r < rows_total) {
    // row space: block b = tb * G + hd holds tokens 32 tb .. 32 tb + 31 of head g G + hd
    const uint32_t blk = (uint32_t)(r >> 5), tb = div_g(p, blk);
    const int i = (int)(32 * tb + (r & 31)), h = g * p.G + (int)(blk - tb * p.G);
    const int64_t off = (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride + lane16 * 8;
    const uint4 a = *reinterpret_cast<const uint4*>((const bf16_t*)p.d_o + off);
    const uint4 b = *reinterpret_cast<const uint4*>((const bf16_t*)p.o + off);
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      acc += __uint_as_float(aw[k] << 16) * __uint_as_float(bw[k] << 16);
      acc += __uint_as_float(aw[k] & 0xffff0000u) * __uint_as_float(bw[k] & 0xffff0000u);
    }
    l2 = p.lse[(int64_t)h * p.C + i] * 1.4426950408889634f;
  }
#pragma unroll
  for (int o = 8; o >= 1; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (lane16 == 0) {
    delta_rs[idx] = acc;
    lse2_rs[idx] = l2;
    if (r < rows_total) {
      float* b = bias + (((int64_t)g * n_stages + (r >> 6)) * 2) * 64 + (r & 63);
      b[0] = -l2 / (p.sm_scale * 1.4426950408889634f);
      b[64] = -acc;
    }
  }
}

// ---------------------------------------------------------------------------------
// dQ.  LDS: two stages of {K half tile, V half tile} (64 keys x 128 dims, 16 KiB each, row tiles).
// One barrier per half tile of 64 keys; the next half tile is copied straight from the paged pools
// into the other stage with direct global -> LDS loads while the current one is consumed (the
// swizzle is applied on the source side, so no re-laid-out copy of the pages is needed).  K^T for
// the dQ product is read from the K tile with the transposing LDS read.
constexpr int DQ_LDS = 4 * 16384;

__global__ __launch_bounds__(BW_THREADS) void bwd_dq_kernel(Params p, const float* __restrict__ delta_rs,
                                                            const float* __restrict__ lse2_rs, int64_t rows_pad,
                                                            int tiles_per_head, int xcd_map) {
  extern __shared__ __align__(16) unsigned char smem[];
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const int tid = threadIdx.x, lane = tid & 63, hh = lane >> 5, lq = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int g, tile;
  if (xcd_map) {
    const int xcd = blockIdx.x & 7, per = 8 / p.Hkv;
    g = xcd % p.Hkv;
    tile = (blockIdx.x >> 3) * per + xcd / p.Hkv;
  } else {
    g = blockIdx.x % p.Hkv;
    tile = blockIdx.x / p.Hkv;
  }
  if (tile >= tiles_per_head) return;
  tile = tiles_per_head - 1 - tile;

  // this wave's block of the row space (one head, 32 consecutive tokens) and the tile's page list
  const RowTile rt = row_tile(p, g, tile, wave);
  const int lid = rt.lid;
  const int64_t first_q = p.N - p.C;
  const bool r_valid = rt.valid;                           // wave-uniform
  const uint32_t bw = rt.bw;
  const uint32_t tbw = div_g(p, bw);
  const int i = (int)(32 * tbw + lq), h = g * p.G + (int)(bw - tbw * p.G);
  const int64_t r = (int64_t)32 * bw + lq;                 // index into the row-space statistics
  const int64_t a_i = first_q + i;
  const int64_t a_wave_max = first_q + 32 * tbw + 31;
  const int64_t a_blk_max = first_q + 32 * div_g(p, (uint32_t)rt.b_last) + 31;

  const int32_t T = visible_len(p, lid, a_blk_max / TP, lane);
  PageWindow pw;
  pw.init(p, lid, T, lane, false);
  int32_t T2 = 2 * T;
  if (T > 0 && (int64_t)list_at(p, lid, T - 1) * TP + 64 > a_blk_max) T2 -= 1;  // second half of the last page unseen
  // half tiles [0, T_full) are seen in full by every row of the workgroup
  int32_t T_full = 0;
  {
    const int64_t a_blk_min = first_q + 32 * (int64_t)div_g(p, (uint32_t)rt.b_first);
    if (a_blk_min >= TP - 1) T_full = 2 * visible_len(p, lid, (a_blk_min - (TP - 1)) / TP, lane);
    if (T_full > T2) T_full = T2;
  }

  const int64_t roff = (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride;
  bf16x8 qf[8], dof[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    qf[kk] = as_bf16x8(*reinterpret_cast<const uint4*>((const bf16_t*)p.q + roff + 16 * kk + 8 * hh));
    dof[kk] = as_bf16x8(*reinterpret_cast<const uint4*>((const bf16_t*)p.d_o + roff + 16 * kk + 8 * hh));
  }
  const float lse2 = lse2_rs[(int64_t)g * rows_pad + r];
  const float dlt = delta_rs[(int64_t)g * rows_pad + r];
  const float c = p.sm_scale * 1.4426950408889634f;

  f32x16 dq[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int x = 0; x < 16; ++x) dq[db][x] = 0.f;

  // LDS operand addresses: (lane base ^ constant) + immediate
  uint32_t na[8], tt[8];
  row_tile_addrs(lq, hh, 0, na);
  row_tile_tr_addrs(lane, 0, tt);

  // Staging.  A half tile of K (and of V) is 64 consecutive tokens of one page and KV head in the
  // pool; wave w moves its rows 8 w .. 8 w + 7 (2 KiB of the LDS tile) with two direct global -> LDS
  // loads per tile: no staging registers, no LDS store instructions.  The kernel waits for them
  // itself before the barrier that publishes the stage.
  uint32_t cp0, cp1;
  row_tile_src_offsets(8 * wave, lane, (uint32_t)(p.pool_tok_stride * 2), cp0, cp1);
  const int64_t head_off = (int64_t)g * p.pool_head_stride;
  auto copy_stage = [&](const int32_t ht, const int st) __attribute__((always_inline)) {
    const int64_t o = ((int64_t)pw.phys(ht >> 1) * p.pool_page_stride + head_off + (int64_t)(ht & 1) * 64 * p.pool_tok_stride) * 2;
    copy_rows_to_lds((const unsigned char*)p.k_pool + o, cp0, cp1, st * 32768 + 2048 * wave);
    copy_rows_to_lds((const unsigned char*)p.v_pool + o, cp0, cp1, st * 32768 + 16384 + 2048 * wave);
  };
  auto copies_landed = [&]() __attribute__((always_inline)) { wait_copies<0>(); };
  auto ht_first = [&](int32_t ht) -> int64_t { return (int64_t)pw.page(ht >> 1) * TP + (ht & 1) * 64; };

  // One half tile is 12 batches of four matrix instructions.  Per 32-key block kb2: four batches
  // compute S^T and dP^T (fragments: K rows and V rows of k-steps 2b, 2b+1, used alternately so
  // that neighbouring instructions are independent), the vector unit turns them into dS^T, and two
  // batches add K^T dS^T of the block to dQ^T (dim blocks 0,1 then 2,3; transposing reads of the K
  // tile, two per fragment).  The fragments of a batch are fetched while the previous batch
  // computes; one wait per batch.
  u32x4 fr[8];
  bf16x8 dsf[2];
  auto fetch = [&](const int st, const int n, const int set) __attribute__((always_inline)) {
    const int kb2 = n / 6, b = n % 6;
    const int o = st * 32768 + kb2 * 8192;
    if (b < 4) {
      fr[set + 0] = *reinterpret_cast<const u32x4*>(smem + (na[2 * b] + o));
      fr[set + 1] = *reinterpret_cast<const u32x4*>(smem + (na[2 * b] + (o + 16384)));
      fr[set + 2] = *reinterpret_cast<const u32x4*>(smem + (na[2 * b + 1] + o));
      fr[set + 3] = *reinterpret_cast<const u32x4*>(smem + (na[2 * b + 1] + (o + 16384)));
    } else {
      const int db = 2 * (b - 4);
      fr[set + 0] = row_tile_tr_frag(smem, tt[2 * db], tt[2 * db + 1], o);
      fr[set + 1] = row_tile_tr_frag(smem, tt[2 * db + 2], tt[2 * db + 3], o);
      fr[set + 2] = row_tile_tr_frag(smem, tt[2 * db], tt[2 * db + 1], o + 4096);
      fr[set + 3] = row_tile_tr_frag(smem, tt[2 * db + 2], tt[2 * db + 3], o + 4096);
    }
  };
  auto half_tile = [&](const int st, const bool general, const int rel) __attribute__((always_inline)) {
    f32x16 sv, dp;
    fetch(st, 0, 0);
#pragma unroll
    for (int n = 0; n < 12; ++n) {
      const int set = 4 * (n & 1);
      const int kb2 = n / 6, b = n % 6;
      if (n + 1 < 12) {
        fetch(st, n + 1, 4 - set);
        // this batch has arrived: only the reads of the next one (4 row reads or 8 transposing reads) are out
        if ((n + 1) % 6 < 4) __builtin_amdgcn_s_waitcnt(0xC47F);  // lgkmcnt(4)
        else __builtin_amdgcn_s_waitcnt(0xC87F);                  // lgkmcnt(8)
        __builtin_amdgcn_sched_barrier(0);   // keep the fetch ahead of this batch's matrix instructions
      }
      if (b < 4) {
        if (b == 0) {
#pragma unroll
          for (int x = 0; x < 16; ++x) { sv[x] = 0.f; dp[x] = 0.f; }
        }
        sv = mfma32(__builtin_bit_cast(bf16x8, fr[set + 0]), qf[2 * b], sv);
        dp = mfma32(__builtin_bit_cast(bf16x8, fr[set + 1]), dof[2 * b], dp);
        sv = mfma32(__builtin_bit_cast(bf16x8, fr[set + 2]), qf[2 * b + 1], sv);
        dp = mfma32(__builtin_bit_cast(bf16x8, fr[set + 3]), dof[2 * b + 1], dp);
        __builtin_amdgcn_sched_barrier(0);
        if (b == 3) {  // dS^T = P^T o (dP^T - Delta) of this 32-key block, rounded to bf16
#pragma unroll
          for (int x = 0; x < 16; ++x) {
            float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[x], c, -lse2));
            if (general && 32 * kb2 + 8 * (x >> 2) + (x & 3) > rel) pr = 0.f;
            sv[x] = pr * (dp[x] - dlt);
          }
          dsf[0] = as_bf16x8(pack8(sv, 0));
          dsf[1] = as_bf16x8(pack8(sv, 8));
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
        const int db = 2 * (b - 4);
        dq[db] = mfma32(__builtin_bit_cast(bf16x8, fr[set + 0]), dsf[0], dq[db]);
        dq[db + 1] = mfma32(__builtin_bit_cast(bf16x8, fr[set + 1]), dsf[0], dq[db + 1]);
        dq[db] = mfma32(__builtin_bit_cast(bf16x8, fr[set + 2]), dsf[1], dq[db]);
        dq[db + 1] = mfma32(__builtin_bit_cast(bf16x8, fr[set + 3]), dsf[1], dq[db + 1]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  if (T2 > 0) copy_stage(0, 0);
  copies_landed();
  __syncthreads();

  // st = t mod 2 is a compile-time constant: the loops are unrolled by two.  The copy of the next
  // half tile goes to the other stage, whose readers finished before the last barrier.
  auto iteration = [&](const int32_t t, const int st, const bool general) __attribute__((always_inline)) {
    pw.advance(p, lid, T, t >> 1, lane);
    if (t + 1 < T2) copy_stage(t + 1, st ^ 1);
    if (!r_valid) {
      // a wave without a block of its own (last row tile of a query page) only moves data and keeps the barriers
    } else if (!general) {
      half_tile(st, false, 0);
    } else {
      const int64_t kfirst = ht_first(t);
      if (kfirst <= a_wave_max)  // wave-uniform: some row of this wave sees the half tile
        half_tile(st, true, (int)(a_i - kfirst) - 4 * hh);  // key index (without the 4 hh term) must be <= rel
    }
    copies_landed();
    __syncthreads();
  };
  {
    int32_t t = 0;
    for (; t + 2 <= T_full; t += 2) {
      iteration(t, 0, false);
      iteration(t + 1, 1, false);
    }
    for (; t < T2; t += 2) {
      iteration(t, 0, true);
      if (t + 1 < T2) iteration(t + 1, 1, true);
    }
  }

  if (r_valid) {
    bf16_t* orow = (bf16_t*)p.d_q + roff;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        uint2 w;
        w.x = pack2_bf16(dq[db][4 * a + 0] * p.sm_scale, dq[db][4 * a + 1] * p.sm_scale);
        w.y = pack2_bf16(dq[db][4 * a + 2] * p.sm_scale, dq[db][4 * a + 3] * p.sm_scale);
        *reinterpret_cast<uint2*>(orow + 32 * db + 8 * a + 4 * hh) = w;
      }
  }
}

static inline size_t stats_bytes(const Params& p) {
  return (2 * (size_t)p.Hkv * (size_t)rows_padded(p) * sizeof(float) + 255) & ~(size_t)255;
}
static inline int32_t row_stages(const Params& p) { return (p.C / 32) * p.G / 2; }   // 64-row stages of the dK/dV kernel
static inline size_t bias_bytes(const Params& p) { return (size_t)p.Hkv * (size_t)row_stages(p) * 512; }

size_t bwd_mfma_workspace_bytes(const Params& p, int32_t max_list_len) {
  return stats_bytes(p) + bias_bytes(p) + dkv_partial_bytes(p, max_list_len, dkv_splits(p, max_list_len));
}

hipError_t launch_bwd_mfma(const Params& p, int32_t max_list_len, void* ws, hipStream_t st) {
  static DeviceOnce lds_once;
  if (hipError_t e = ensure_max_dynamic_lds(lds_once, (const void*)bwd_dq_kernel, DQ_LDS); e != hipSuccess) return e;
  const int64_t rows_pad = rows_padded(p);
  float* delta_rs = (float*)ws;
  float* lse2_rs = delta_rs + (size_t)p.Hkv * rows_pad;
  float* bias = (float*)((unsigned char*)ws + stats_bytes(p));   // bias words of the dK/dV kernel
  {
    const int64_t total = (int64_t)p.Hkv * rows_pad;
    ProfScope prof_("bwd_prep", st);
    bwd_prep_kernel<<<dim3((unsigned)((total + 15) / 16)), dim3(256), 0, st>>>(p, delta_rs, lse2_rs, rows_pad, bias,
                                                                               row_stages(p));
  }
  const int xcd_map = (p.Hkv <= 8 && 8 % p.Hkv == 0) ? 1 : 0;
  const int per = xcd_map ? 8 / p.Hkv : 1;
  {
    const int tiles = row_tiles_per_head(p.C, p.G, p.m, p.qp);
    const unsigned blocks = xcd_map ? 8u * (unsigned)((tiles + per - 1) / per) : (unsigned)tiles * p.Hkv;
    ProfScope prof_("bwd_dq_mfma", st);
    bwd_dq_kernel<<<dim3(blocks), dim3(BW_THREADS), DQ_LDS, st>>>(p, delta_rs, lse2_rs, rows_pad, tiles, xcd_map);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_bwd_dkv_mfma(p, bias, row_stages(p), max_list_len, (float*)((unsigned char*)bias + bias_bytes(p)), st);
}

}  // namespace oomb
