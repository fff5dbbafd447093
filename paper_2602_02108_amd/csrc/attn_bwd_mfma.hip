// Paged attention backward with bf16 MFMA (paper Sec. 3 Eq. 3 and Sec. 4.1: dK/dV
// are accumulated in place into the paged gradient pool; Sec. 4.2: the forward's
// page list is reused).  Page size 128, head dim 128.
//
// Three kernels:
//   bwd_prep : Delta = <dO, O> and LSE * log2(e), both re-laid out in the KV head's
//              "row space" r = i * G + (h - g * G) and padded to whole tiles.
//   bwd_dq   : parallel over 256-row tiles (like the forward); per half page of 64
//              keys: S^T = K Q^T, dP^T = V dO^T, dS^T = P^T o (dP^T - Delta),
//              dQ^T += K^T dS^T.  Every lane owns one query row.
//   bwd_dkv  : one workgroup OWNS one (KV head, selected page): it visits every query
//              row that sees the page, accumulates dK^T and dV^T in registers and
//              read-modify-writes the page of the gradient pool once, with plain
//              loads and stores.  No atomics; results do not depend on scheduling.
#include "mfma_common.h"

namespace oomb {

constexpr int BW_WAVES = 8;
constexpr int BW_THREADS = BW_WAVES * 64;
constexpr int DQ_ROWS = 256;
constexpr int ROW_PAD = 256;  // row-space statistics are padded to a multiple of this

// swizzled byte offset inside a tile whose rows hold GR granules of 16 bytes
template <int GR> __device__ __forceinline__ int toff(int r, int c) {
  return (r * GR + (c ^ (GR == 16 ? (r & 15) : ((r >> 1) & 7)))) * 16;
}
template <int GR> __device__ __forceinline__ bf16x8 lds_frag(const unsigned char* tile, int r, int c) {
  return as_bf16x8(*reinterpret_cast<const uint4*>(tile + toff<GR>(r, c)));
}

__device__ __forceinline__ uint4 pack8(const f32x16& v, int base) {
  uint4 w;
  w.x = pack2_bf16(v[base + 0], v[base + 1]);
  w.y = pack2_bf16(v[base + 2], v[base + 3]);
  w.z = pack2_bf16(v[base + 4], v[base + 5]);
  w.w = pack2_bf16(v[base + 6], v[base + 7]);
  return w;
}

__device__ __forceinline__ uint4 pack_hi_lo(const uint32_t* r, uint32_t sel) {
  uint4 w;
  w.x = __builtin_amdgcn_perm(r[1], r[0], sel);
  w.y = __builtin_amdgcn_perm(r[3], r[2], sel);
  w.z = __builtin_amdgcn_perm(r[5], r[4], sel);
  w.w = __builtin_amdgcn_perm(r[7], r[6], sel);
  return w;
}

static inline int64_t rows_padded(const Params& p) {
  const int64_t rows = (int64_t)p.C * p.G;
  return (rows + ROW_PAD - 1) / ROW_PAD * ROW_PAD;
}

// ---------------------------------------------------------------------------------
// 16 lanes per row (8 elements each), 4 rows per wave.
__global__ __launch_bounds__(256) void bwd_prep_kernel(Params p, float* __restrict__ delta_rs,
                                                       float* __restrict__ lse2_rs, int64_t rows_pad) {
  const int lane16 = threadIdx.x & 15;
  const int64_t idx = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);  // over Hkv * rows_pad
  if (idx >= (int64_t)p.Hkv * rows_pad) return;
  const int g = (int)(idx / rows_pad);
  const int64_t r = idx % rows_pad;
  const int64_t rows_total = (int64_t)p.C * p.G;
  float acc = 0.f, l2 = 1e30f;
  if (r < rows_total) {
    const int i = (int)(r / p.G), h = g * p.G + (int)(r % p.G);
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
  }
}

// ---------------------------------------------------------------------------------
// dQ.  LDS: two stages of {K natural half tile, V natural half tile, K transposed
// half tile}, 16 KiB each.
constexpr int DQ_STAGE = 3 * 16384;
constexpr int DQ_LDS = 2 * DQ_STAGE;

struct DqStage {
  uint4 kn[2], vn[2];
  uint32_t kt[8];
  // half tile hf of the page at kb / vb
  __device__ __forceinline__ void load(const bf16_t* kb, const bf16_t* vb, int64_t ts, int hf, int tid, int wave,
                                       int lane) {
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const int gi = tid + BW_THREADS * x;
      const int64_t o = (int64_t)(64 * hf + (gi >> 4)) * ts + (gi & 15) * 8;
      kn[x] = *reinterpret_cast<const uint4*>(kb + o);
      vn[x] = *reinterpret_cast<const uint4*>(vb + o);
    }
    const int u = wave >> 1, h2 = wave & 1;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int tok = 64 * hf + 16 * u + 4 * h2 + (e & 3) + 8 * (e >> 2);
      kt[e] = *reinterpret_cast<const uint32_t*>(kb + (int64_t)tok * ts + 2 * lane);
    }
  }
  __device__ __forceinline__ void store(unsigned char* st, int tid, int wave, int lane) const {
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const int gi = tid + BW_THREADS * x;
      *reinterpret_cast<uint4*>(st + toff<16>(gi >> 4, gi & 15)) = kn[x];
      *reinterpret_cast<uint4*>(st + 16384 + toff<16>(gi >> 4, gi & 15)) = vn[x];
    }
    *reinterpret_cast<uint4*>(st + 32768 + toff<8>(2 * lane, wave)) = pack_hi_lo(kt, 0x05040100u);
    *reinterpret_cast<uint4*>(st + 32768 + toff<8>(2 * lane + 1, wave)) = pack_hi_lo(kt, 0x07060302u);
  }
};

__global__ __launch_bounds__(BW_THREADS) void bwd_dq_kernel(Params p, const float* __restrict__ delta_rs,
                                                            const float* __restrict__ lse2_rs, int64_t rows_pad,
                                                            int tiles_per_head, int xcd_map) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hh = lane >> 5, lq = lane & 31;
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

  const int64_t rows_total = (int64_t)p.C * p.G;
  const int64_t row0 = (int64_t)tile * DQ_ROWS;
  const int64_t first_q = p.N - p.C;
  const int64_t r_raw = row0 + wave * 32 + lq;
  const bool r_valid = r_raw < rows_total;
  const int64_t r = r_valid ? r_raw : rows_total - 1;
  const int i = (int)(r / p.G), h = g * p.G + (int)(r % p.G);
  const int64_t a_i = first_q + i;
  const int64_t rw_lo = row0 + wave * 32, rw_hi_raw = rw_lo + 31;
  const int64_t rw_hi = rw_hi_raw < rows_total ? rw_hi_raw : rows_total - 1;
  const int64_t a_wave_min = first_q + (rw_lo < rows_total ? rw_lo : rows_total - 1) / p.G;
  const int64_t a_wave_max = first_q + rw_hi / p.G;
  const int64_t rb_hi = (row0 + DQ_ROWS - 1 < rows_total) ? row0 + DQ_ROWS - 1 : rows_total - 1;
  const int64_t a_blk_max = first_q + rb_hi / p.G;

  int32_t T = list_len(p, g);
  {
    const int64_t l_max = a_blk_max / TP;
    while (T > 0 && list_at(p, g, T - 1) > l_max) --T;
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

  DqStage stg;
  auto tile_ptrs = [&](int32_t j, const bf16_t*& kb, const bf16_t*& vb, int64_t& first) {
    const int64_t l = list_at(p, g, j);
    const int64_t off = (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride;
    kb = (const bf16_t*)p.k_pool + off;
    vb = (const bf16_t*)p.v_pool + off;
    first = l * TP;
  };
  const bf16_t *kb = nullptr, *vb = nullptr;
  int64_t first = 0, first_cur = 0;
  const int32_t n_st = 2 * T;
  if (n_st > 0) {
    tile_ptrs(0, kb, vb, first);
    stg.load(kb, vb, p.pool_tok_stride, 0, tid, wave, lane);
    stg.store(smem, tid, wave, lane);
  }
  __syncthreads();

  for (int32_t st = 0; st < n_st; ++st) {
    const int b = st & 1, hf = st & 1;  // stage parity doubles as the half index
    const unsigned char* sb = smem + b * DQ_STAGE;
    first_cur = first;
    if (st + 1 < n_st) {
      if (((st + 1) & 1) == 0) tile_ptrs((st + 1) >> 1, kb, vb, first);
      stg.load(kb, vb, p.pool_tok_stride, (st + 1) & 1, tid, wave, lane);
    }
    const int64_t kfirst = first_cur + 64 * hf;
    if (kfirst <= a_wave_max) {
      const bool diag = kfirst + 63 > a_wave_min;
      bf16x8 dsf[4];
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2) {
        f32x16 s, dp;
#pragma unroll
        for (int x = 0; x < 16; ++x) { s[x] = 0.f; dp[x] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
          s = mfma32(lds_frag<16>(sb, 32 * kb2 + lq, 2 * kk + hh), qf[kk], s);
          dp = mfma32(lds_frag<16>(sb + 16384, 32 * kb2 + lq, 2 * kk + hh), dof[kk], dp);
        }
#pragma unroll
        for (int x = 0; x < 16; ++x) {
          float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(s[x], c, -lse2));
          if (diag) {
            const int64_t key = kfirst + 32 * kb2 + 8 * (x >> 2) + 4 * hh + (x & 3);
            if (key > a_i) pr = 0.f;
          }
          s[x] = pr * (dp[x] - dlt);
        }
        dsf[2 * kb2 + 0] = as_bf16x8(pack8(s, 0));
        dsf[2 * kb2 + 1] = as_bf16x8(pack8(s, 8));
      }
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int u = 0; u < 4; ++u)
          dq[db] = mfma32(lds_frag<8>(sb + 32768, 32 * db + lq, 2 * u + hh), dsf[u], dq[db]);
    }
    if (st + 1 < n_st) stg.store(smem + (b ^ 1) * DQ_STAGE, tid, wave, lane);
    __syncthreads();
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

// ---------------------------------------------------------------------------------
// dK / dV.  LDS: V natural tile (32 KiB) + two stages of {Q natural, dO natural,
// Q transposed, dO transposed} for 64 query rows, 16 KiB each  (160 KiB in all).
constexpr int KV_STAGE = 4 * 16384;
constexpr int KV_LDS = TILE_BYTES + 2 * KV_STAGE;

struct KvStage {
  uint4 qn[2], don[2];
  uint32_t qt[8], dot[8];
  // 64 rows of row space starting at R0
  __device__ __forceinline__ void load(const Params& p, int g, uint32_t R0, uint32_t rows_total, int tid, int wave,
                                       int lane) {
    const bf16_t* q = (const bf16_t*)p.q;
    const bf16_t* d_o = (const bf16_t*)p.d_o;
    const int64_t hbase = (int64_t)g * p.G * p.q_head_stride;
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const int gi = tid + BW_THREADS * x;
      const uint32_t rr = R0 + (gi >> 4);
      if (rr < rows_total) {
        const uint32_t i = div_g(p, rr), hd = rr - i * p.G;
        const int64_t o = (int64_t)i * p.q_tok_stride + hbase + (int64_t)hd * p.q_head_stride + (gi & 15) * 8;
        qn[x] = *reinterpret_cast<const uint4*>(q + o);
        don[x] = *reinterpret_cast<const uint4*>(d_o + o);
      } else {
        qn[x] = make_uint4(0, 0, 0, 0);
        don[x] = make_uint4(0, 0, 0, 0);
      }
    }
    const int u = wave >> 1, h2 = wave & 1;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t rr = R0 + 16 * u + 4 * h2 + (e & 3) + 8 * (e >> 2);  // wave-uniform
      if (rr < rows_total) {
        const uint32_t i = div_g(p, rr), hd = rr - i * p.G;
        const int64_t o = (int64_t)i * p.q_tok_stride + hbase + (int64_t)hd * p.q_head_stride + 2 * lane;
        qt[e] = *reinterpret_cast<const uint32_t*>(q + o);
        dot[e] = *reinterpret_cast<const uint32_t*>(d_o + o);
      } else {
        qt[e] = 0;
        dot[e] = 0;
      }
    }
  }
  __device__ __forceinline__ void store(unsigned char* st, int tid, int wave, int lane) const {
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const int gi = tid + BW_THREADS * x;
      *reinterpret_cast<uint4*>(st + toff<16>(gi >> 4, gi & 15)) = qn[x];
      *reinterpret_cast<uint4*>(st + 16384 + toff<16>(gi >> 4, gi & 15)) = don[x];
    }
    *reinterpret_cast<uint4*>(st + 32768 + toff<8>(2 * lane, wave)) = pack_hi_lo(qt, 0x05040100u);
    *reinterpret_cast<uint4*>(st + 32768 + toff<8>(2 * lane + 1, wave)) = pack_hi_lo(qt, 0x07060302u);
    *reinterpret_cast<uint4*>(st + 49152 + toff<8>(2 * lane, wave)) = pack_hi_lo(dot, 0x05040100u);
    *reinterpret_cast<uint4*>(st + 49152 + toff<8>(2 * lane + 1, wave)) = pack_hi_lo(dot, 0x07060302u);
  }
};

template <typename TG>
__device__ __forceinline__ void rmw4(TG* ptr, float a, float b, float c2, float d);
template <>
__device__ __forceinline__ void rmw4<float>(float* ptr, float a, float b, float c2, float d) {
  float4 v = *reinterpret_cast<float4*>(ptr);
  v.x += a; v.y += b; v.z += c2; v.w += d;
  *reinterpret_cast<float4*>(ptr) = v;
}
template <>
__device__ __forceinline__ void rmw4<bf16_t>(bf16_t* ptr, float a, float b, float c2, float d) {
  uint2 v = *reinterpret_cast<uint2*>(ptr);
  uint2 w;
  w.x = pack2_bf16(__uint_as_float(v.x << 16) + a, __uint_as_float(v.x & 0xffff0000u) + b);
  w.y = pack2_bf16(__uint_as_float(v.y << 16) + c2, __uint_as_float(v.y & 0xffff0000u) + d);
  *reinterpret_cast<uint2*>(ptr) = w;
}

template <typename TG>
__global__ __launch_bounds__(BW_THREADS) void bwd_dkv_kernel(Params p, const float* __restrict__ delta_rs,
                                                             const float* __restrict__ lse2_rs, int64_t rows_pad,
                                                             int32_t max_len, int xcd_map) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hh = lane >> 5, lq = lane & 31;
  const int kbw = wave & 3, qh = wave >> 2;
  int g;
  int32_t j;
  if (xcd_map) {
    const int xcd = blockIdx.x & 7, per = 8 / p.Hkv;
    g = xcd % p.Hkv;
    j = (blockIdx.x >> 3) * per + xcd / p.Hkv;
  } else {
    g = blockIdx.x % p.Hkv;
    j = blockIdx.x / p.Hkv;
  }
  if (j >= max_len || j >= list_len(p, g)) return;

  const int64_t rows_total = (int64_t)p.C * p.G;
  const int64_t first_q = p.N - p.C;
  const int64_t l = list_at(p, g, j);
  const int64_t first = l * TP;
  const int64_t pool_off = (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride;
  const bf16_t* kb = (const bf16_t*)p.k_pool + pool_off;
  const bf16_t* vb = (const bf16_t*)p.v_pool + pool_off;
  const float c = p.sm_scale * 1.4426950408889634f;

  // this wave's 32 keys as the B operand of S = Q K^T, kept in registers
  bf16x8 kf[8];
  {
    const bf16_t* krow = kb + (int64_t)(32 * kbw + lq) * p.pool_tok_stride;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) kf[kk] = as_bf16x8(*reinterpret_cast<const uint4*>(krow + 16 * kk + 8 * hh));
  }
  unsigned char* vt = smem;
  unsigned char* stages = smem + TILE_BYTES;
  {
    NaturalStage<BW_THREADS> vst;
    vst.load(vb, p.pool_tok_stride, tid);
    vst.store(vt, tid);
  }

  // first row that sees this page, rounded down to a stage boundary
  const int64_t r_start = (first > first_q ? first - first_q : 0) * p.G;
  const int64_t s0 = r_start / 64, s_end = (rows_total + 63) / 64;

  f32x16 dkt[4], dvt[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int x = 0; x < 16; ++x) { dkt[db][x] = 0.f; dvt[db][x] = 0.f; }

  KvStage stg;
  if (s0 < s_end) {
    stg.load(p, g, (uint32_t)(s0 * 64), (uint32_t)rows_total, tid, wave, lane);
    stg.store(stages, tid, wave, lane);
  }
  __syncthreads();

  const int64_t key_pos = first + 32 * kbw + lq;
  for (int64_t s = s0; s < s_end; ++s) {
    const int b = (int)((s - s0) & 1);
    const unsigned char* sb = stages + b * KV_STAGE;
    if (s + 1 < s_end) stg.load(p, g, (uint32_t)((s + 1) * 64), (uint32_t)rows_total, tid, wave, lane);

    const int64_t R0 = s * 64 + 32 * qh;  // first row of this wave's 32-query block
    f32x16 sc, dp;
#pragma unroll
    for (int x = 0; x < 16; ++x) { sc[x] = 0.f; dp[x] = 0.f; }
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      sc = mfma32(lds_frag<16>(sb, 32 * qh + lq, 2 * kk + hh), kf[kk], sc);
      dp = mfma32(lds_frag<16>(sb + 16384, 32 * qh + lq, 2 * kk + hh), lds_frag<16>(vt, 32 * kbw + lq, 2 * kk + hh), dp);
    }
    const bool diag = first_q + div_g(p, (uint32_t)R0) < first + TP - 1;  // some (row, key) of the block may be masked
    const float* l2p = lse2_rs + (int64_t)g * rows_pad + R0 + 4 * hh;
    const float* dlp = delta_rs + (int64_t)g * rows_pad + R0 + 4 * hh;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const float4 l2 = *reinterpret_cast<const float4*>(l2p + 8 * a);
      const float4 dl = *reinterpret_cast<const float4*>(dlp + 8 * a);
      const float l2v[4] = {l2.x, l2.y, l2.z, l2.w}, dlv[4] = {dl.x, dl.y, dl.z, dl.w};
#pragma unroll
      for (int bb = 0; bb < 4; ++bb) {
        const int x = 4 * a + bb;
        float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[x], c, -l2v[bb]));
        if (diag) {
          const int64_t row = R0 + 8 * a + 4 * hh + bb;
          if (key_pos > first_q + div_g(p, (uint32_t)row)) pr = 0.f;
        }
        sc[x] = pr;
        dp[x] = pr * (dp[x] - dlv[bb]);
      }
    }
    bf16x8 pf[2], dsf[2];
    pf[0] = as_bf16x8(pack8(sc, 0));
    pf[1] = as_bf16x8(pack8(sc, 8));
    dsf[0] = as_bf16x8(pack8(dp, 0));
    dsf[1] = as_bf16x8(pack8(dp, 8));
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        dvt[db] = mfma32(lds_frag<8>(sb + 49152, 32 * db + lq, 2 * (2 * qh + u) + hh), pf[u], dvt[db]);
        dkt[db] = mfma32(lds_frag<8>(sb + 32768, 32 * db + lq, 2 * (2 * qh + u) + hh), dsf[u], dkt[db]);
      }

    if (s + 1 < s_end) stg.store(stages + (b ^ 1) * KV_STAGE, tid, wave, lane);
    __syncthreads();
  }

  // combine the two query halves: waves qh = 0 finish dK, waves qh = 1 finish dV
  float* xch = reinterpret_cast<float*>(stages);  // 8 slots of 16 KiB
  {
    const f32x16* give = (qh == 0) ? dvt : dkt;
    float* slot = xch + (size_t)wave * 4096;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int x4 = 0; x4 < 4; ++x4) {
        float4 v = {give[db][4 * x4 + 0], give[db][4 * x4 + 1], give[db][4 * x4 + 2], give[db][4 * x4 + 3]};
        *reinterpret_cast<float4*>(slot + ((db * 4 + x4) * 64 + lane) * 4) = v;
      }
  }
  __syncthreads();
  {
    f32x16* mine = (qh == 0) ? dkt : dvt;
    const float* slot = xch + (size_t)(wave ^ 4) * 4096;
    const float scale = (qh == 0) ? p.sm_scale : 1.f;
    TG* pool = (TG*)((qh == 0) ? p.dk_pool : p.dv_pool) + pool_off + (int64_t)(32 * kbw + lq) * p.pool_tok_stride;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const float4 o = *reinterpret_cast<const float4*>(slot + ((db * 4 + a) * 64 + lane) * 4);
        rmw4<TG>(pool + 32 * db + 8 * a + 4 * hh, (mine[db][4 * a + 0] + o.x) * scale, (mine[db][4 * a + 1] + o.y) * scale,
                 (mine[db][4 * a + 2] + o.z) * scale, (mine[db][4 * a + 3] + o.w) * scale);
      }
  }
}

size_t bwd_mfma_workspace_bytes(const Params& p, int32_t) {
  return 2 * (size_t)p.Hkv * (size_t)rows_padded(p) * sizeof(float);
}

hipError_t launch_bwd_mfma(const Params& p, int32_t max_list_len, void* ws, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)bwd_dq_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, DQ_LDS);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void*)bwd_dkv_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, KV_LDS);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void*)bwd_dkv_kernel<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, KV_LDS);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int64_t rows_pad = rows_padded(p);
  float* delta_rs = (float*)ws;
  float* lse2_rs = delta_rs + (size_t)p.Hkv * rows_pad;
  {
    const int64_t total = (int64_t)p.Hkv * rows_pad;
    ProfScope prof_("bwd_prep", st);
    bwd_prep_kernel<<<dim3((unsigned)((total + 15) / 16)), dim3(256), 0, st>>>(p, delta_rs, lse2_rs, rows_pad);
  }
  const int xcd_map = (p.Hkv <= 8 && 8 % p.Hkv == 0) ? 1 : 0;
  const int per = xcd_map ? 8 / p.Hkv : 1;
  {
    const int tiles = (int)(((int64_t)p.C * p.G + DQ_ROWS - 1) / DQ_ROWS);
    const unsigned blocks = xcd_map ? 8u * (unsigned)((tiles + per - 1) / per) : (unsigned)tiles * p.Hkv;
    ProfScope prof_("bwd_dq_mfma", st);
    bwd_dq_kernel<<<dim3(blocks), dim3(BW_THREADS), DQ_LDS, st>>>(p, delta_rs, lse2_rs, rows_pad, tiles, xcd_map);
  }
  {
    const unsigned blocks = xcd_map ? 8u * (unsigned)((max_list_len + per - 1) / per) : (unsigned)max_list_len * p.Hkv;
    ProfScope prof_("bwd_dkv_mfma", st);
    if (p.grad_is_bf16)
      bwd_dkv_kernel<bf16_t><<<dim3(blocks), dim3(BW_THREADS), KV_LDS, st>>>(p, delta_rs, lse2_rs, rows_pad, max_list_len, xcd_map);
    else
      bwd_dkv_kernel<float><<<dim3(blocks), dim3(BW_THREADS), KV_LDS, st>>>(p, delta_rs, lse2_rs, rows_pad, max_list_len, xcd_map);
  }
  return hipGetLastError();
}

}  // namespace oomb
