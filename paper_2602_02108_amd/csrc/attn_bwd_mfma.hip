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

  // row space: block b = tb * G + hd holds tokens 32 tb .. 32 tb + 31 of head g G + hd;
  // wave w of tile t owns block 8 t + w
  const int32_t nblk = (p.C / 32) * p.G;
  const int64_t first_q = p.N - p.C;
  const int32_t b_raw = tile * (DQ_ROWS / 32) + wave;
  const bool r_valid = b_raw < nblk;                       // wave-uniform
  const uint32_t bw = (uint32_t)(r_valid ? b_raw : nblk - 1);
  const uint32_t tbw = div_g(p, bw);
  const int i = (int)(32 * tbw + lq), h = g * p.G + (int)(bw - tbw * p.G);
  const int64_t r = (int64_t)32 * bw + lq;                 // index into the row-space statistics
  const int64_t a_i = first_q + i;
  const int64_t a_wave_min = first_q + 32 * tbw, a_wave_max = a_wave_min + 31;
  const int32_t b_last = (tile * (DQ_ROWS / 32) + 7 < nblk) ? tile * (DQ_ROWS / 32) + 7 : nblk - 1;
  const int64_t a_blk_max = first_q + 32 * div_g(p, (uint32_t)b_last) + 31;

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

size_t dkv_partial_bytes(const Params& p, int32_t max_len, int32_t n_split);
int32_t dkv_splits(const Params& p, int32_t max_len);
hipError_t launch_bwd_dkv_mfma(const Params& p, const float* delta_rs, const float* lse2_rs, int64_t rows_pad,
                               int32_t max_len, float* partial_ws, hipStream_t st);

static inline size_t stats_bytes(const Params& p) {
  return (2 * (size_t)p.Hkv * (size_t)rows_padded(p) * sizeof(float) + 255) & ~(size_t)255;
}

size_t bwd_mfma_workspace_bytes(const Params& p, int32_t max_list_len) {
  return stats_bytes(p) + dkv_partial_bytes(p, max_list_len, dkv_splits(p, max_list_len));
}

hipError_t launch_bwd_mfma(const Params& p, int32_t max_list_len, void* ws, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)bwd_dq_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, DQ_LDS);
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
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_bwd_dkv_mfma(p, delta_rs, lse2_rs, rows_pad, max_list_len, (float*)((char*)ws + stats_bytes(p)), st);
}

}  // namespace oomb
