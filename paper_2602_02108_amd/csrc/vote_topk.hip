// Retrieval by voting (paper Sec. 4.2, the scoring equation): every query token scores
// all key pages against their mean keys, the scores become a distribution over the key
// pages (softmax along the key-page index), the distributions of the tokens of a query
// page -- and of the G query heads that share the KV head -- are summed into one vote per
// key page, and every query page keeps its top-K pages.
//
// The logits are a dense contraction, rows (C G per KV head) x pages (n_past) x D, so they
// run on the matrix cores (bf16 operands: the page means are rounded to bf16 once), in two
// passes over row tiles of 8 blocks of 32 rows (the row space of the attention kernels):
//   pass 1  S^T = Kbar Q^T: a lane owns a query row; online max / sum -> log2-sum-exp per row
//   pass 2  S = Q Kbar^T (operands swapped, same fragments): a lane owns a page column and
//           16 rows; p = exp2(c S - lse2[row]) summed down the column, then over the 8 waves
//           in a fixed order -> one partial vote per (row tile, page); a tile whose rows belong
//           to two query pages keeps two partial votes, one per query page
// then the partial votes of a query page's row tiles are added (fixed order) and the top-K
// selection kernel runs once per (KV head, query page).  No atomics: bit-reproducible.
// Shapes without a matrix kernel (fp32 tensors, D or P != 128) take two plain kernels.
#include "mfma_common.h"
#include "launch.h"

namespace oomb {

constexpr int VT_THREADS = 512;
constexpr int VT_RED = 2 * 16384;            // cross-wave reduction buffers behind the two Kbar buffers
constexpr int VT_LDS = VT_RED + 2 * 8 * 64 * 4;

static inline size_t vt_up(size_t x) { return (x + 255) & ~(size_t)255; }

// ---- images of the page means -------------------------------------------------------------------
// Kbar of KV head g, rounded to bf16, as natural half tiles of 64 pages x 128 dims in the byte
// order of the LDS tile (page r of the half tile, granule c at (r * 16 + (c ^ (r & 15))) * 16);
// pages at and beyond n_past are zero rows.
__global__ __launch_bounds__(256) void kbar_image_kernel(Params p, const float* __restrict__ kbar,
                                                         unsigned char* __restrict__ img, int32_t n_ht) {
  const int ht = blockIdx.x, g = blockIdx.y, tid = threadIdx.x;
  unsigned char* out = img + ((size_t)g * n_ht + ht) * 16384;
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    const int gi = tid + 256 * x, r = gi >> 4, cg = gi & 15;
    const int64_t l = (int64_t)64 * ht + r;
    uint4 w = make_uint4(0, 0, 0, 0);
    if (l < p.n_past) {
      const float4* src = reinterpret_cast<const float4*>(kbar + ((size_t)l * p.Hkv + g) * HD + 8 * cg);
      const float4 a = src[0], b = src[1];
      w.x = (uint32_t)f32_to_bf16(a.x) | ((uint32_t)f32_to_bf16(a.y) << 16);
      w.y = (uint32_t)f32_to_bf16(a.z) | ((uint32_t)f32_to_bf16(a.w) << 16);
      w.z = (uint32_t)f32_to_bf16(b.x) | ((uint32_t)f32_to_bf16(b.y) << 16);
      w.w = (uint32_t)f32_to_bf16(b.z) | ((uint32_t)f32_to_bf16(b.w) << 16);
    }
    *reinterpret_cast<uint4*>(out + (r * 16 + (cg ^ (r & 15))) * 16) = w;
  }
}

// ---- the two passes -----------------------------------------------------------------------------
// PASS = 1: lse2_rs[g][row] = log2 sum over past pages of exp2(c * logit), row-space index.
// PASS = 2: part[((g tiles + tile) 2 + k) n_pad + page] = sum over the rows of the tile that belong to
//           its first (k = 0) / second (k = 1) query page of exp2(c * logit - lse2[row]).
template <int PASS>
__global__ __launch_bounds__(VT_THREADS) void vote_pass_kernel(Params p, const unsigned char* __restrict__ kb_img,
                                                               int32_t n_ht, float* __restrict__ lse2_rs, int64_t rows_pad,
                                                               int tiles_per_head, int xcd_map, float* __restrict__ part,
                                                               int64_t n_pad) {
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

  const RowTile rt = row_tile(p, g, tile, wave);  // (p.qp is clear: the tiles partition the row space)
  // query page of a block: b / bpq.  The waves from `split` on belong to the tile's second query page.
  const int32_t bpq = (p.P / 32) * p.G;
  const int32_t tau_lo = rt.b_first / bpq;
  const int32_t split = rt.b_last / bpq != tau_lo ? (tau_lo + 1) * bpq - rt.b_first : 8;
  const uint32_t bw = rt.bw, tbw = div_g(p, bw);
  const int i = (int)(32 * tbw + lq), h = g * p.G + (int)(bw - tbw * p.G);
  const bf16_t* qrow = (const bf16_t*)p.q + (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride;
  bf16x8 qf[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) qf[kk] = as_bf16x8(*reinterpret_cast<const uint4*>(qrow + 16 * kk + 8 * hh));
  const float c = p.sm_scale * 1.4426950408889634f;

  uint32_t ka[8];
  {
    const uint32_t kbase = lq * 256 + (((lq & 15) ^ hh) << 4);
#pragma unroll
    for (int j = 0; j < 8; ++j) ka[j] = kbase ^ (j << 5);
  }
  const unsigned char* const img_g = kb_img + (size_t)g * n_ht * 16384;
  const uint32_t cp_off = 2048 * wave + 16 * lane;
  auto copy_ht = [&](int32_t ht, const int buf) __attribute__((always_inline)) {
    copy_kib_to_lds<2>(img_g + (size_t)ht * 16384, cp_off, buf * 16384 + 2048 * wave);
  };

  // pass 1 state: per-lane row statistics; pass 2 state: lse2 of the 16 rows this lane holds
  float m_run = -1e30f, l_run = 0.f;
  float lse_r[16];
  if (PASS == 2) {
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      const int row = 8 * (x >> 2) + 4 * hh + (x & 3);
      lse_r[x] = rt.valid ? lse2_rs[(int64_t)g * rows_pad + (int64_t)32 * bw + row] : INFINITY;  // idle waves vote 0
    }
  }
  float* const part_t = PASS == 2 ? part + ((int64_t)g * tiles_per_head + tile) * 2 * n_pad : nullptr;

  if (n_ht > 0) copy_ht(0, 0);
  wait_copies<0>();
  __syncthreads();

  auto iteration = [&](const int32_t t, const int buf) __attribute__((always_inline)) {
    if (t + 1 < n_ht) copy_ht(t + 1, buf ^ 1);
    // (a wave without a block of its own only moves data and keeps the barriers; in pass 2 it votes 0)
    if (!rt.valid) {
      if (PASS == 2 && hh == 0) {
        *reinterpret_cast<float*>(smem + (VT_RED + ((buf * 8 + wave) * 64 + lq) * 4)) = 0.f;
        *reinterpret_cast<float*>(smem + (VT_RED + ((buf * 8 + wave) * 64 + 32 + lq) * 4)) = 0.f;
      }
    } else {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        f32x16 s;
#pragma unroll
        for (int x = 0; x < 16; ++x) s[x] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(smem + (ka[j] + (buf * 16384 + u * 8192))));
          s = PASS == 1 ? mfma32(kf, qf[j], s) : mfma32(qf[j], kf, s);
        }
        if (PASS == 1) {
          // s[x]: page 64 t + 32 u + 8 (x / 4) + 4 hh + x % 4, this lane's row
          if (t == n_ht - 1) {
            const int64_t first = (int64_t)64 * t + 32 * u + 4 * hh;
#pragma unroll
            for (int x = 0; x < 16; ++x)
              if (first + 8 * (x >> 2) + (x & 3) >= p.n_past) s[x] = -INFINITY;
          }
          float mx = s[0];
#pragma unroll
          for (int x = 1; x < 16; ++x) mx = fmaxf(mx, s[x]);
          mx = half_max(mx);
          const float m_new = fmaxf(m_run, mx);
          const float mc = m_new * c;
          float sum = 0.f;
#pragma unroll
          for (int x = 0; x < 16; ++x) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(s[x], c, -mc));
          l_run = l_run * __builtin_amdgcn_exp2f((m_run - m_new) * c) + sum;
          m_run = m_new;
        } else {
          // s[x]: row 8 (x / 4) + 4 hh + x % 4 of this wave, page 64 t + 32 u + lq
          float col = 0.f;
#pragma unroll
          for (int x = 0; x < 16; ++x) col += __builtin_amdgcn_exp2f(__builtin_fmaf(s[x], c, -lse_r[x]));
          col = half_sum(col);
          if (hh == 0) *reinterpret_cast<float*>(smem + (VT_RED + ((buf * 8 + wave) * 64 + 32 * u + lq) * 4)) = col;
        }
      }
    }
    wait_copies<0>();
    __syncthreads();
    if (PASS == 2 && wave == (t & 7)) {
      // votes of half tile t: the waves' column sums, added in wave order, per query page of the tile
      float v0 = 0.f, v1 = 0.f;
#pragma unroll
      for (int w = 0; w < 8; ++w) {
        const float x = *reinterpret_cast<const float*>(smem + (VT_RED + ((buf * 8 + w) * 64 + lane) * 4));
        if (w < split) v0 += x;
        else v1 += x;
      }
      const int64_t page = (int64_t)64 * t + lane;
      if (page < p.n_past) {
        part_t[page] = v0;
        if (split < 8) part_t[n_pad + page] = v1;
      }
    }
  };
  for (int32_t t = 0; t < n_ht; t += 2) {
    iteration(t, 0);
    if (t + 1 < n_ht) iteration(t + 1, 1);
  }

  if (PASS == 1) {
    const float l_tot = half_sum(l_run);
    if (rt.valid && hh == 0)
      lse2_rs[(int64_t)g * rows_pad + (int64_t)32 * bw + lq] = m_run * c + __builtin_amdgcn_logf(l_tot);
  }
}

// votes[g][tau][l] = sum over the row tiles that hold rows of the query page (ascending) of their
// partial votes for it
__global__ __launch_bounds__(256) void vote_finish_kernel(const float* __restrict__ part, float* __restrict__ votes,
                                                          int64_t n_past, int64_t n_pad, int32_t tiles, int32_t m, int32_t bpq) {
  const int64_t l = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int32_t q = blockIdx.y, g = q / m, tau = q - g * m;
  if (l >= n_past) return;
  float v = 0.f;
  for (int32_t t = tau * bpq / 8; t <= ((tau + 1) * bpq - 1) / 8; ++t) {
    const int32_t k = (8 * t) / bpq == tau ? 0 : 1;  // the tile's first or second query page
    v += part[(((int64_t)g * tiles + t) * 2 + k) * n_pad + l];
  }
  votes[(int64_t)q * n_past + l] = v;
}

// ---- shapes without a matrix kernel ---------------------------------------------------------------
// One wave per query row: natural-log-sum-exp of its logits over the past pages.
template <typename T>
__global__ __launch_bounds__(256) void vote_lse_generic_kernel(Params p, const float* __restrict__ kbar, int round_bf16,
                                                               float* __restrict__ lse) {
  __shared__ float qs[4][128];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * 4 + w;
  if (row >= (int64_t)p.C * p.Hq) return;
  const int i = (int)(row / p.Hq), h = (int)(row % p.Hq), g = h / p.G;
  const T* qrow = (const T*)p.q + (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride;
  for (int d = lane; d < p.D; d += 64) qs[w][d] = Elem<T>::load(qrow + d);
  __builtin_amdgcn_wave_barrier();
  float m_run = -INFINITY, l_run = 0.f;
  for (int64_t l = lane; l < p.n_past; l += 64) {
    const float* kb = kbar + ((size_t)l * p.Hkv + g) * p.D;
    float dot = 0.f;
    for (int d = 0; d < p.D; ++d) dot += qs[w][d] * (round_bf16 ? bf16_to_f32(f32_to_bf16(kb[d])) : kb[d]);
    const float z = p.sm_scale * dot;
    const float m_new = fmaxf(m_run, z);
    l_run = l_run * __expf(m_run - m_new) + __expf(z - m_new);
    m_run = m_new;
  }
  float m_all = m_run;
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) m_all = fmaxf(m_all, __shfl_xor(m_all, o, 64));
  float part = m_run == -INFINITY ? 0.f : l_run * __expf(m_run - m_all);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) part += __shfl_xor(part, o, 64);
  if (lane == 0) lse[(int64_t)h * p.C + i] = m_all + __logf(part);
}

// One thread per (KV head, query page, past page): the rows of the query page in a fixed order.
template <typename T>
__global__ __launch_bounds__(256) void vote_sum_generic_kernel(Params p, const float* __restrict__ kbar, int round_bf16,
                                                               const float* __restrict__ lse, float* __restrict__ votes) {
  const int64_t l = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int tau = blockIdx.y, g = blockIdx.z;
  if (l >= p.n_past) return;
  const float* kb = kbar + ((size_t)l * p.Hkv + g) * p.D;
  float v = 0.f;
  for (int h = g * p.G; h < g * p.G + p.G; ++h)
    for (int i = tau * p.P; i < tau * p.P + p.P; ++i) {
      const T* qrow = (const T*)p.q + (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride;
      float dot = 0.f;
      for (int d = 0; d < p.D; ++d) dot += Elem<T>::load(qrow + d) * (round_bf16 ? bf16_to_f32(f32_to_bf16(kb[d])) : kb[d]);
      v += __expf(p.sm_scale * dot - lse[(int64_t)h * p.C + i]);
    }
  votes[((int64_t)g * p.m + tau) * p.n_past + l] = v;
}

// ---- host side ----------------------------------------------------------------------------------

struct VoteLayout {
  int32_t n_ht, tpq;
  int64_t rows_pad, n_pad;
  size_t off_img, off_lse, off_part, off_votes, bytes;
};

static VoteLayout vote_layout(const Params& p, bool mfma) {
  VoteLayout L{};
  const int64_t np1 = p.n_past > 0 ? p.n_past : 1;
  L.n_ht = (int32_t)((p.n_past + 63) / 64);
  L.n_pad = (int64_t)(L.n_ht > 0 ? L.n_ht : 1) * 64;
  L.tpq = mfma ? row_tiles_per_head(p.C, p.G, p.m, 0) : 1;  // row tiles per KV head
  L.rows_pad = ((int64_t)p.C * p.G + 255) / 256 * 256;
  size_t o = 0;
  auto take = [&](size_t b) { const size_t at = o; o += vt_up(b); return at; };
  L.off_img = take(mfma ? (size_t)p.Hkv * (L.n_ht > 0 ? L.n_ht : 1) * 16384 : 0);
  L.off_lse = take(mfma ? (size_t)p.Hkv * L.rows_pad * 4 : (size_t)p.Hq * p.C * 4);
  L.off_part = take(mfma ? (size_t)p.Hkv * L.tpq * 2 * L.n_pad * 4 : 0);
  L.off_votes = take((size_t)p.Hkv * p.m * np1 * 4);
  L.bytes = o;
  return L;
}

size_t vote_workspace_bytes(const Params& p, bool is_bf16, bool force_generic) {
  return vote_layout(p, !force_generic && mfma_supported(p, is_bf16)).bytes;
}

hipError_t launch_vote_topk(Params p, bool is_bf16, bool force_generic, const float* kbar, int32_t top_k, int32_t* sel,
                            int32_t* sel_count, float* votes_out, void* ws, hipStream_t st) {
  const bool mfma = !force_generic && mfma_supported(p, is_bf16);
  const VoteLayout L = vote_layout(p, mfma);
  unsigned char* b = (unsigned char*)ws;
  float* votes = votes_out ? votes_out : (float*)(b + L.off_votes);
  p.qp = 0;
  if (p.n_past > 0 && mfma) {
    static DeviceOnce lds_once_1, lds_once_2;
    if (hipError_t e = ensure_max_dynamic_lds(lds_once_1, (const void*)vote_pass_kernel<1>, VT_LDS); e != hipSuccess) return e;
    if (hipError_t e = ensure_max_dynamic_lds(lds_once_2, (const void*)vote_pass_kernel<2>, VT_LDS); e != hipSuccess) return e;
    unsigned char* img = b + L.off_img;
    float* lse2 = (float*)(b + L.off_lse);
    float* part = (float*)(b + L.off_part);
    {
      ProfScope prof_("kbar_image", st);
      kbar_image_kernel<<<dim3((unsigned)L.n_ht, (unsigned)p.Hkv), dim3(256), 0, st>>>(p, kbar, img, L.n_ht);
    }
    const int tiles = L.tpq;
    const int xcd_map = (p.Hkv <= 8 && 8 % p.Hkv == 0) ? 1 : 0;
    const int per = xcd_map ? 8 / p.Hkv : 1;
    const unsigned blocks = xcd_map ? 8u * (unsigned)((tiles + per - 1) / per) : (unsigned)tiles * p.Hkv;
    {
      ProfScope prof_("vote_lse", st);
      vote_pass_kernel<1><<<dim3(blocks), dim3(VT_THREADS), VT_LDS, st>>>(p, img, L.n_ht, lse2, L.rows_pad, tiles, xcd_map,
                                                                          nullptr, L.n_pad);
    }
    {
      ProfScope prof_("vote_sum", st);
      vote_pass_kernel<2><<<dim3(blocks), dim3(VT_THREADS), VT_LDS, st>>>(p, img, L.n_ht, lse2, L.rows_pad, tiles, xcd_map,
                                                                          part, L.n_pad);
    }
    {
      ProfScope prof_("vote_finish", st);
      vote_finish_kernel<<<dim3((unsigned)((p.n_past + 255) / 256), (unsigned)(p.Hkv * p.m)), dim3(256), 0, st>>>(
          part, votes, p.n_past, L.n_pad, tiles, p.m, (p.P / 32) * p.G);
    }
  } else if (p.n_past > 0) {
    float* lse = (float*)(b + L.off_lse);
    const int round_bf16 = is_bf16 ? 1 : 0;
    const int64_t rows = (int64_t)p.C * p.Hq;
    dim3 g1((unsigned)((rows + 3) / 4)), g2((unsigned)((p.n_past + 255) / 256), (unsigned)p.m, (unsigned)p.Hkv);
    ProfScope prof_("vote_generic", st);
    if (is_bf16) {
      vote_lse_generic_kernel<bf16_t><<<g1, dim3(256), 0, st>>>(p, kbar, round_bf16, lse);
      vote_sum_generic_kernel<bf16_t><<<g2, dim3(256), 0, st>>>(p, kbar, round_bf16, lse, votes);
    } else {
      vote_lse_generic_kernel<float><<<g1, dim3(256), 0, st>>>(p, kbar, round_bf16, lse);
      vote_sum_generic_kernel<float><<<g2, dim3(256), 0, st>>>(p, kbar, round_bf16, lse, votes);
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_topk_select_qp(p, votes, top_k, sel, sel_count, st);
}

}  // namespace oomb
