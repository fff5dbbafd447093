// Paged attention forward with bf16 MFMA (paper Sec. 4.1 operator over the
// selected pages of Sec. 4.2), page size 128, head dim 128.
//
// A workgroup of 8 waves owns 8 consecutive blocks of one KV head's "row space":
// block b = tb * G + hd is the 32 consecutive chunk tokens 32 tb .. 32 tb + 31 of
// query head g G + hd, i.e. the G query heads of the group interleaved block by
// block, so the K/V tiles staged in LDS are shared by all query heads of the
// group and a workgroup's rows span at most three token blocks (short causal
// diagonal).  Each wave keeps its 32 query rows (as the B operand of
// S^T = K Q^T) and its 32 x 128 output block in registers.  Pages are processed
// as two half tiles of 64 keys: K as a natural half tile, V as a transposed half
// tile, both double buffered and staged through registers.  In
// the S^T layout every lane owns one query row, so the online-softmax
// statistics are per-lane scalars.
//
// Schedule (one barrier per half tile t): S_t = K_t Q^T, online softmax, then
// O += V_t P_t.  LDS operand fragments are fetched in batches of four, one batch
// ahead of the matrix instructions that use them; the next half tile is fetched
// from global memory into registers at the top of an iteration and written to
// the other LDS buffer at its bottom.
#include "mfma_common.h"

namespace oomb {

constexpr int FW_WAVES = 8;
constexpr int FW_THREADS = FW_WAVES * 64;
constexpr int FW_ROWS = FW_WAVES * 32;
constexpr int HT = 64;                    // keys per half tile
constexpr int HT_BYTES = HT * HD * 2;     // 16 KiB
constexpr int FW_LDS = 4 * HT_BYTES;      // K0 K1 V0 V1

__global__ __launch_bounds__(FW_THREADS) void fwd_mfma_kernel(Params p, int tiles_per_head, int xcd_map) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, hh = lane >> 5, lq = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  
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

  // row space: block b = tb * G + hd holds tokens 32 tb .. 32 tb + 31 of head g G + hd;
  // wave w of tile t owns block 8 t + w (one head, 32 consecutive tokens)
  const int32_t nblk = (p.C / 32) * p.G;
  const int64_t first_q = p.N - p.C;
  const int32_t b_raw = tile * (FW_ROWS / 32) + wave;
  const bool r_valid = b_raw < nblk;                       // wave-uniform
  const uint32_t bw = (uint32_t)(r_valid ? b_raw : nblk - 1);
  const uint32_t tbw = div_g(p, bw);
  const uint32_t i = 32 * tbw + lq;
  const int h = g * p.G + (int)(bw - tbw * p.G);
  const int64_t a_i = first_q + i;
  const int64_t a_wave_min = first_q + 32 * tbw, a_wave_max = a_wave_min + 31;
  const int32_t b_last = (tile * (FW_ROWS / 32) + 7 < nblk) ? tile * (FW_ROWS / 32) + 7 : nblk - 1;
  const int64_t a_blk_max = first_q + 32 * div_g(p, (uint32_t)b_last) + 31;

  // number of half tiles visible to this workgroup (lists are ascending)
  const int32_t T = visible_len(p, g, a_blk_max / TP, lane);
  PageWindow pw;
  pw.init(p, g, T, lane);
  int32_t T2 = 2 * T;
  if (T > 0 && (int64_t)list_at(p, g, T - 1) * TP + HT > a_blk_max) T2 -= 1;  // second half of the last page unseen

  const bf16_t* qrow = (const bf16_t*)p.q + (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride;
  bf16x8 qf[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) qf[kk] = as_bf16x8(*reinterpret_cast<const uint4*>(qrow + 16 * kk + 8 * hh));

  f32x16 of[4], sc[2];
  bf16x8 pf[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int x = 0; x < 16; ++x) of[db][x] = 0.f;
#pragma unroll
  for (int u = 0; u < 4; ++u) pf[u] = as_bf16x8(make_uint4(0, 0, 0, 0));
  float m_run = -1e30f, l_run = 0.f;
  const float c = p.sm_scale * 1.4426950408889634f;
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

  // LDS operand addresses.  The swizzles XOR a per-lane constant into the granule
  // index, so an operand address is (lane base ^ small constant) + block offset; the
  // block offset goes into the instruction's immediate field.
  uint32_t ka[8], va[4];
  {
    const uint32_t kbase = lq * 256 + (((lq & 15) ^ hh) << 4);           // natural, 16 granules per row
    const uint32_t vbase = lq * 128 + ((((lq >> 1) & 7) ^ hh) << 4);     // transposed, 8 granules per row
#pragma unroll
    for (int j = 0; j < 8; ++j) ka[j] = kbase ^ (j << 5);
#pragma unroll
    for (int j = 0; j < 4; ++j) va[j] = vbase ^ (j << 5);
  }
  unsigned char* const kbuf = smem;
  unsigned char* const vbuf = smem + 2 * HT_BYTES;

  // half tile ht: page j = ht / 2, keys 64 (ht % 2) .. + 63 of it
  auto ht_first = [&](int32_t ht) -> int64_t { return (int64_t)pw.page(ht >> 1) * TP + (ht & 1) * HT; };
  auto ht_off = [&](int32_t ht) -> int64_t {
    return (int64_t)pw.phys(ht >> 1) * p.pool_page_stride + (int64_t)g * p.pool_head_stride +
           (int64_t)(ht & 1) * HT * p.pool_tok_stride;
  };
  // this wave's share of a K half tile: 8 rows = two 4-row chunks, staged through registers
  // (a direct global -> LDS load makes the compiler wait for it before the next LDS read,
  // which exposes the whole memory latency every iteration).  Lane l of a chunk lands at
  // granule position l % 16 of row l / 16, so it fetches the granule the swizzle maps there.
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 kr0, kr1;
  uint32_t knat_off[2];
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    const uint32_t srow = 8 * wave + 4 * x + (lane >> 4);
    knat_off[x] = srow * ((uint32_t)p.pool_tok_stride * 2u) + (((lane & 15) ^ (srow & 15)) << 4);
  }
  auto load_k = [&](int32_t ht) {
    const char* base = reinterpret_cast<const char*>((const bf16_t*)p.k_pool + ht_off(ht));
    kr0 = *reinterpret_cast<const u32x4*>(base + knat_off[0]);
    kr1 = *reinterpret_cast<const u32x4*>(base + knat_off[1]);
  };
  auto store_k = [&](unsigned char* dst) {
    *reinterpret_cast<u32x4*>(dst + (8 * wave) * 256 + lane * 16) = kr0;
    *reinterpret_cast<u32x4*>(dst + (8 * wave + 4) * 256 + lane * 16) = kr1;
  };
  // this wave's octet (index = wave) of a V half tile: tokens 16u + 4h2 + {0..3, 8..11}
  uint32_t vr[8], vro[8];
  {
    const int u = wave >> 1, h2 = wave & 1;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      vro[e] = (uint32_t)(16 * u + 4 * h2 + (e & 3) + 8 * (e >> 2)) * ((uint32_t)p.pool_tok_stride * 2u) + (uint32_t)lane * 4u;
  }
  auto load_v = [&](int32_t ht) {
    const char* base = reinterpret_cast<const char*>((const bf16_t*)p.v_pool + ht_off(ht));
#pragma unroll
    for (int e = 0; e < 8; ++e) vr[e] = *reinterpret_cast<const uint32_t*>(base + vro[e]);
  };
  auto store_v = [&](unsigned char* dst) {
    uint4 lo, hi;
    lo.x = __builtin_amdgcn_perm(vr[1], vr[0], 0x05040100u);
    lo.y = __builtin_amdgcn_perm(vr[3], vr[2], 0x05040100u);
    lo.z = __builtin_amdgcn_perm(vr[5], vr[4], 0x05040100u);
    lo.w = __builtin_amdgcn_perm(vr[7], vr[6], 0x05040100u);
    hi.x = __builtin_amdgcn_perm(vr[1], vr[0], 0x07060302u);
    hi.y = __builtin_amdgcn_perm(vr[3], vr[2], 0x07060302u);
    hi.z = __builtin_amdgcn_perm(vr[5], vr[4], 0x07060302u);
    hi.w = __builtin_amdgcn_perm(vr[7], vr[6], 0x07060302u);
    const int d0 = 2 * lane, d1 = 2 * lane + 1;
    *reinterpret_cast<uint4*>(dst + (d0 * 8 + (wave ^ ((d0 >> 1) & 7))) * 16) = lo;
    *reinterpret_cast<uint4*>(dst + (d1 * 8 + (wave ^ ((d1 >> 1) & 7))) * 16) = hi;
  };
  // S^T (64 keys x 32 queries) = K Q^T; fragments fetched one batch of four ahead
  auto qk = [&](f32x16* dst, const unsigned char* kt) {
    uint4 fa[4], fb[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) fa[j] = *reinterpret_cast<const uint4*>(kt + ka[j]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 4; ++j) fb[j] = *reinterpret_cast<const uint4*>(kt + ka[4 + j]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int x = 0; x < 16; ++x) { dst[0][x] = 0.f; dst[1][x] = 0.f; }
#pragma unroll
    for (int j = 0; j < 4; ++j) dst[0] = mfma32(as_bf16x8(fa[j]), qf[j], dst[0]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 4; ++j) fa[j] = *reinterpret_cast<const uint4*>(kt + ka[j] + 8192);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 4; ++j) dst[0] = mfma32(as_bf16x8(fb[j]), qf[4 + j], dst[0]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 4; ++j) fb[j] = *reinterpret_cast<const uint4*>(kt + ka[4 + j] + 8192);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 4; ++j) dst[1] = mfma32(as_bf16x8(fa[j]), qf[j], dst[1]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 4; ++j) dst[1] = mfma32(as_bf16x8(fb[j]), qf[4 + j], dst[1]);
    __builtin_amdgcn_sched_barrier(0);
  };
  // O^T (128 dims x 32 queries) += V^T P^T
  auto pv = [&](const unsigned char* vt) {
    uint4 fa[4], fb[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) fa[u] = *reinterpret_cast<const uint4*>(vt + va[u]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 4; ++u) fb[u] = *reinterpret_cast<const uint4*>(vt + va[u] + 4096);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 4; ++u) of[0] = mfma32(as_bf16x8(fa[u]), pf[u], of[0]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 4; ++u) fa[u] = *reinterpret_cast<const uint4*>(vt + va[u] + 2 * 4096);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 4; ++u) of[1] = mfma32(as_bf16x8(fb[u]), pf[u], of[1]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 4; ++u) fb[u] = *reinterpret_cast<const uint4*>(vt + va[u] + 3 * 4096);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 4; ++u) of[2] = mfma32(as_bf16x8(fa[u]), pf[u], of[2]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 4; ++u) of[3] = mfma32(as_bf16x8(fb[u]), pf[u], of[3]);
    __builtin_amdgcn_sched_barrier(0);
  };
  // causal mask of a diagonal half tile (first token `first`)
  auto mask_diag = [&](f32x16* sv, int64_t first) {
    const int rel = (int)(a_i - first) - 4 * hh;  // key index (without the 4 hh term) must be <= rel
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
      for (int x = 0; x < 16; ++x)
        if (32 * kb2 + 8 * (x >> 2) + (x & 3) > rel) sv[kb2][x] = -INFINITY;
  };
  auto row_max = [&](const f32x16* sv) -> float {
    float mx = sv[0][0];
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
      for (int x = 0; x < 16; ++x) mx = fmaxf(mx, sv[kb2][x]);
    return half_max(mx);
  };
  // m_run <- max(m_run, m_tile); O and l are rescaled only when some row's maximum moved
  auto rescale = [&](float m_tile) {
    const float m_new = fmaxf(m_run, m_tile);
    if (__any(m_new != m_run)) {  // wave-uniform
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int x = 0; x < 16; ++x) of[db][x] *= alpha;
      m_run = m_new;
    }
  };
  // P = exp2(c S - c m_run) of the half tile in sc, rounded to bf16 into pf; returns the
  // row sum of the rounded probabilities (what the PV product uses)
  auto exps = [&]() -> float {
    const float mc = m_run * c;
    float rs = 0.f;
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2) {
#pragma unroll
      for (int x = 0; x < 16; ++x) sc[kb2][x] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kb2][x], c, -mc));
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        uint4 w;
        w.x = pack2_bf16(sc[kb2][8 * u + 0], sc[kb2][8 * u + 1]);
        w.y = pack2_bf16(sc[kb2][8 * u + 2], sc[kb2][8 * u + 3]);
        w.z = pack2_bf16(sc[kb2][8 * u + 4], sc[kb2][8 * u + 5]);
        w.w = pack2_bf16(sc[kb2][8 * u + 6], sc[kb2][8 * u + 7]);
        rs = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.x), ones, rs, false);
        rs = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.y), ones, rs, false);
        rs = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.z), ones, rs, false);
        rs = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.w), ones, rs, false);
        pf[2 * kb2 + u] = as_bf16x8(w);
      }
    }
    return rs;
  };

  // prologue: K_0 and V_0 into LDS
  if (T2 > 0) {
    load_k(0);
    load_v(0);
    store_k(kbuf);
    store_v(vbuf);
  }
  __syncthreads();
  // Half tiles [0, T_full) are seen in full by every row of the workgroup: their loop body is
  // straight-line code with no masking and no per-wave conditions.  The remaining (diagonal)
  // half tiles run the general body.  V buffers alternate like the K buffers.
  int32_t T_full = 0;
  {
    const int64_t a_blk_min = first_q + 32 * (int64_t)div_g(p, (uint32_t)(tile * (FW_ROWS / 32)));
    if (a_blk_min >= TP - 1) T_full = 2 * visible_len(p, g, (a_blk_min - (TP - 1)) / TP, lane);
    if (T_full > T2) T_full = T2;
  }
  auto iteration = [&](const int32_t t, const bool general) {
    pw.advance(p, g, T, t >> 1, lane);
    const bool more = t + 1 < T2;
    if (more) {
      load_k(t + 1);
      load_v(t + 1);
    }
    const unsigned char* kt = kbuf + (t & 1) * HT_BYTES;
    const unsigned char* vt = vbuf + (t & 1) * HT_BYTES;
    if (!general) {
      qk(sc, kt);
      rescale(row_max(sc));
      l_run += exps();
      pv(vt);
    } else {
      const int64_t first = ht_first(t);
      if (first <= a_wave_max) {  // wave-uniform: some row of this wave sees the half tile
        qk(sc, kt);
        if (first + HT - 1 > a_wave_min) mask_diag(sc, first);
        rescale(row_max(sc));
        l_run += exps();
        pv(vt);
      }
    }
    if (more) {
      store_k(kbuf + ((t + 1) & 1) * HT_BYTES);
      store_v(vbuf + ((t + 1) & 1) * HT_BYTES);
    }
    __syncthreads();
  };
  for (int32_t t = 0; t < T_full; ++t) iteration(t, false);
  for (int32_t t = T_full; t < T2; ++t) iteration(t, true);

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
  { ProfScope prof_("attn_fwd_mfma", st); fwd_mfma_kernel<<<dim3(blocks), dim3(FW_THREADS), FW_LDS, st>>>(p, tiles, xcd_map); }
  return hipGetLastError();
}

}  // namespace oomb
