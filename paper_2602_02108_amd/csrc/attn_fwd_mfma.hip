// Paged attention forward with bf16 MFMA (paper Sec. 4.1 operator over the
// selected pages of Sec. 4.2), page size 128, head dim 128.
//
// A workgroup of 8 waves owns 256 consecutive rows of one KV head's "row space":
// row r = i * G + (h - g * G), i.e. the G query heads of the group interleaved
// token by token, so the K/V tiles staged in LDS are shared by all query heads
// of the group and a workgroup's rows span only 256 / G tokens (short causal
// diagonal).  Each wave keeps its 32 query rows (as the B operand of
// S^T = K Q^T) and its 32 x 128 output block in registers; K is staged as a
// natural tile, V as a transposed tile (see mfma_common.h), double buffered.
// In the S^T layout every lane owns one query row, so the online-softmax
// statistics are per-lane scalars.
#include "mfma_common.h"

namespace oomb {

constexpr int FW_WAVES = 8;
constexpr int FW_THREADS = FW_WAVES * 64;
constexpr int FW_ROWS = FW_WAVES * 32;
constexpr int FW_LDS = 4 * TILE_BYTES;  // K0 K1 V0 V1

__global__ __launch_bounds__(FW_THREADS) void fwd_mfma_kernel(Params p, int tiles_per_head, int xcd_map) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hh = lane >> 5, lq = lane & 31;

  // workgroup -> (KV head, row tile).  Workgroups are dealt round-robin to the 8
  // XCDs; keeping a KV head on a fixed set of XCDs lets its pages stay in that L2.
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
  tile = tiles_per_head - 1 - tile;  // rows late in the chunk see more local pages: start them first

  const int64_t rows_total = (int64_t)p.C * p.G;
  const int64_t row0 = (int64_t)tile * FW_ROWS;
  const int64_t first_q = p.N - p.C;

  // this lane's query row
  const int64_t r_raw = row0 + wave * 32 + lq;
  const bool r_valid = r_raw < rows_total;
  const int64_t r = r_valid ? r_raw : rows_total - 1;
  const int i = (int)(r / p.G), h = g * p.G + (int)(r % p.G);
  const int64_t a_i = first_q + i;
  // wave-uniform bounds of the wave's rows (for skipping / masking decisions)
  const int64_t rw_lo = row0 + wave * 32, rw_hi_raw = rw_lo + 31;
  const int64_t rw_hi = rw_hi_raw < rows_total ? rw_hi_raw : rows_total - 1;
  const int64_t a_wave_min = first_q + (rw_lo < rows_total ? rw_lo : rows_total - 1) / p.G;
  const int64_t a_wave_max = first_q + rw_hi / p.G;
  const int64_t rb_hi = (row0 + FW_ROWS - 1 < rows_total) ? row0 + FW_ROWS - 1 : rows_total - 1;
  const int64_t a_blk_max = first_q + rb_hi / p.G;

  // number of list entries visible to this workgroup (lists are ascending)
  int32_t T = list_len(p, g);
  {
    const int64_t l_max = a_blk_max / TP;
    while (T > 0 && list_at(p, g, T - 1) > l_max) --T;
  }

  const bf16_t* qrow = (const bf16_t*)p.q + (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride;
  bf16x8 qf[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) qf[kk] = as_bf16x8(*reinterpret_cast<const uint4*>(qrow + 16 * kk + 8 * hh));

  f32x16 of[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int x = 0; x < 16; ++x) of[db][x] = 0.f;
  float m_run = -1e30f, l_run = 0.f;
  const float c = p.sm_scale * 1.4426950408889634f;

  NaturalStage<FW_THREADS> ks;
  TransposedStage<FW_WAVES> vs;
  auto tile_ptrs = [&](int32_t j, const bf16_t*& kb, const bf16_t*& vb, int64_t& first) {
    const int64_t l = list_at(p, g, j);
    const int64_t off = (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride;
    kb = (const bf16_t*)p.k_pool + off;
    vb = (const bf16_t*)p.v_pool + off;
    first = l * TP;
  };

  const bf16_t *kb, *vb;
  int64_t first = 0, first_next = 0;
  if (T > 0) {
    tile_ptrs(0, kb, vb, first);
    ks.load(kb, p.pool_tok_stride, tid);
    vs.load(vb, p.pool_tok_stride, wave, lane);
    ks.store(smem, tid);
    vs.store(smem + 2 * TILE_BYTES, wave, lane);
  }
  __syncthreads();

  for (int32_t j = 0; j < T; ++j) {
    const int b = j & 1;
    const unsigned char* kt = smem + b * TILE_BYTES;
    const unsigned char* vt = smem + (2 + b) * TILE_BYTES;
    const bool more = j + 1 < T;
    if (more) {
      tile_ptrs(j + 1, kb, vb, first_next);
      ks.load(kb, p.pool_tok_stride, tid);
      vs.load(vb, p.pool_tok_stride, wave, lane);
    }

    if (first <= a_wave_max) {  // wave-uniform: some row of this wave sees the tile
      // S^T = K Q^T : 4 key blocks of 32, contraction over the head dim in 8 steps
      f32x16 s[4];
#pragma unroll
      for (int kbk = 0; kbk < 4; ++kbk) {
#pragma unroll
        for (int x = 0; x < 16; ++x) s[kbk][x] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
          s[kbk] = mfma32(as_bf16x8(lds_read16(kt, 32 * kbk + lq, 2 * kk + hh)), qf[kk], s[kbk]);
      }
      if (first + TP - 1 > a_wave_min) {  // diagonal tile: mask keys after the query
#pragma unroll
        for (int kbk = 0; kbk < 4; ++kbk)
#pragma unroll
          for (int x = 0; x < 16; ++x) {
            const int64_t key = first + 32 * kbk + 8 * (x >> 2) + 4 * hh + (x & 3);
            if (key > a_i) s[kbk][x] = -INFINITY;
          }
      }
      float mx = s[0][0];
#pragma unroll
      for (int kbk = 0; kbk < 4; ++kbk)
#pragma unroll
        for (int x = 0; x < 16; ++x) mx = fmaxf(mx, s[kbk][x]);
      mx = half_max(mx);
      const float m_new = fmaxf(m_run, mx);
      const float mc = m_new * c;
      float rs = 0.f;
      bf16x8 pf[8];
#pragma unroll
      for (int kbk = 0; kbk < 4; ++kbk) {
#pragma unroll
        for (int x = 0; x < 16; ++x) {
          s[kbk][x] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kbk][x], c, -mc));
          rs += s[kbk][x];
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          uint4 w;
          w.x = pack2_bf16(s[kbk][8 * u + 0], s[kbk][8 * u + 1]);
          w.y = pack2_bf16(s[kbk][8 * u + 2], s[kbk][8 * u + 3]);
          w.z = pack2_bf16(s[kbk][8 * u + 4], s[kbk][8 * u + 5]);
          w.w = pack2_bf16(s[kbk][8 * u + 6], s[kbk][8 * u + 7]);
          pf[2 * kbk + u] = as_bf16x8(w);
        }
      }
      if (__any(m_new != m_run)) {  // wave-uniform: rescale only when some row's maximum moved
        const float alpha = __builtin_amdgcn_exp2f(__builtin_fmaf(m_run, c, -mc));
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int x = 0; x < 16; ++x) of[db][x] *= alpha;
        m_run = m_new;
      }
      l_run += rs;
      // O^T += V^T P^T : 4 head-dim blocks of 32, contraction over 8 groups of 16 keys
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int u = 0; u < 8; ++u)
          of[db] = mfma32(as_bf16x8(lds_read16(vt, 32 * db + lq, 2 * u + hh)), pf[u], of[db]);
    }

    if (more) {
      ks.store(smem + (b ^ 1) * TILE_BYTES, tid);
      vs.store(smem + (2 + (b ^ 1)) * TILE_BYTES, wave, lane);
      first = first_next;
    }
    __syncthreads();
  }

  // epilogue: O = acc / l, LSE = ln(2) * (m * c + log2 l)
  const float l_tot = half_sum(l_run);
  if (r_valid) {
    const float inv = 1.f / l_tot;
    bf16_t* orow = (bf16_t*)p.o + (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        uint2 w;
        w.x = pack2_bf16(of[db][4 * a + 0] * inv, of[db][4 * a + 1] * inv);
        w.y = pack2_bf16(of[db][4 * a + 2] * inv, of[db][4 * a + 3] * inv);
        *reinterpret_cast<uint2*>(orow + 32 * db + 8 * a + 4 * hh) = w;
      }
    if (hh == 0) p.lse[(int64_t)h * p.C + i] = (m_run * c + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
  }
}

bool mfma_supported(const Params& p, bool is_bf16) {
  return is_bf16 && p.D == HD && p.P == TP;
}

hipError_t launch_fwd_mfma(const Params& p, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)fwd_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, FW_LDS);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int64_t rows = (int64_t)p.C * p.G;
  const int tiles = (int)((rows + FW_ROWS - 1) / FW_ROWS);
  const int xcd_map = (p.Hkv <= 8 && 8 % p.Hkv == 0) ? 1 : 0;
  unsigned blocks;
  if (xcd_map) {
    const int per = 8 / p.Hkv;
    blocks = 8u * (unsigned)((tiles + per - 1) / per);
  } else {
    blocks = (unsigned)tiles * p.Hkv;
  }
  fwd_mfma_kernel<<<dim3(blocks), dim3(FW_THREADS), FW_LDS, st>>>(p, tiles, xcd_map);
  return hipGetLastError();
}

}  // namespace oomb
