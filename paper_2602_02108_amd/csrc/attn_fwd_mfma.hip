// Paged attention forward with bf16 MFMA (paper Sec. 4.1 operator over the
// selected pages of Sec. 4.2), page size 128, head dim 128.
//
// A workgroup of 8 waves owns up to 8 consecutive blocks of one KV head's "row space":
// block b = tb * G + hd is the 32 consecutive chunk tokens 32 tb .. 32 tb + 31 of
// query head g G + hd, i.e. the G query heads of the group interleaved block by
// block, so the K/V tiles staged in LDS are shared by all query heads of the
// group and a workgroup's rows span at most three token blocks (short causal
// diagonal).  Each wave keeps its 32 query rows (as the B operand of
// S^T = K Q^T) and its 32 x 128 output block in registers.  In the S^T layout
// every lane owns one query row, so the online-softmax statistics are per-lane
// scalars.
//
// Pages are processed as half tiles of 64 keys -- K natural, V transposed -- that
// are copied verbatim from pre-laid-out images (kv_layout.hip) into three K and
// three V buffers in LDS with direct global -> LDS loads, a whole iteration ahead
// of their use; one barrier per half tile.  The arithmetic runs as a three-stage
// software pipeline over units of 32 keys: O += V_u P_u and S_{u+2} = K_{u+2} Q^T
// on the matrix unit while the vector unit does the online softmax of unit u + 1
// (see "the software pipeline" below).
//
// The page list of a row tile is the KV head's list, or -- one list per query page
// (Sec. 4.2, votes per query page) -- the list of the tile's query page, whose
// entries name their K/V images by position in the union of the head's lists.
#include "mfma_common.h"
#include "launch.h"

namespace oomb {

constexpr int FW_WAVES = 8;
constexpr int FW_THREADS = FW_WAVES * 64;
constexpr int FW_ROWS = FW_WAVES * 32;
constexpr int HT = 64;                    // keys per half tile
constexpr int HT_BYTES = HT * HD * 2;     // 16 KiB
constexpr int FW_LDS = 6 * HT_BYTES;      // K0 K1 K2 V0 V1 V2

__global__ __launch_bounds__(FW_THREADS) void fwd_mfma_kernel(Params p, int tiles_per_head, int xcd_map,
                                                              const unsigned char* __restrict__ k_img,
                                                              const unsigned char* __restrict__ vt_img, int32_t img_len) {
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

  // this wave's block of the row space (one head, 32 consecutive tokens) and the tile's page list
  const RowTile rt = row_tile(p, g, tile, wave);
  const int lid = rt.lid;
  const int64_t first_q = p.N - p.C;
  const bool r_valid = rt.valid;                           // wave-uniform
  const uint32_t bw = rt.bw;
  const uint32_t tbw = div_g(p, bw);
  const uint32_t i = 32 * tbw + lq;
  const int h = g * p.G + (int)(bw - tbw * p.G);
  const int64_t a_i = first_q + i;
  const int64_t a_blk_max = first_q + 32 * div_g(p, (uint32_t)rt.b_last) + 31;

  // number of half tiles visible to this workgroup (lists are ascending)
  const int32_t T = visible_len(p, lid, a_blk_max / TP, lane);
  PageWindow pw;
  pw.init(p, lid, T, lane, p.qp != 0);
  int32_t T2 = 2 * T;
  if (T > 0 && (int64_t)list_at(p, lid, T - 1) * TP + HT > a_blk_max) T2 -= 1;  // second half of the last page unseen

  const bf16_t* qrow = (const bf16_t*)p.q + (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride;
  bf16x8 qf[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) qf[kk] = as_bf16x8(*reinterpret_cast<const uint4*>(qrow + 16 * kk + 8 * hh));

  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  f32x16 of[4], sA, sB;   // output block; scores of the two units in flight
  u32x4 pA[2], pB[2];     // bf16 probabilities of the two units in flight (B operands of V^T P^T)
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int x = 0; x < 16; ++x) of[db][x] = 0.f;
#pragma unroll
  for (int u = 0; u < 2; ++u) { pA[u] = (u32x4){0u, 0u, 0u, 0u}; pB[u] = (u32x4){0u, 0u, 0u, 0u}; }
  float m_run = -1e30f, l_run = 0.f, alpha_pend = 1.f;
  const float c = p.sm_scale * 1.4426950408889634f;
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

  // LDS operand addresses.  The swizzles XOR a per-lane constant into the granule
  // index, so an operand address is (lane base ^ small constant) + block offset; the
  // block offset goes into the instruction's immediate field.
  // LDS: V buffers at 0, 16K, 32K; K buffers at 48K, 64K, 80K.  The K addresses carry the 48K in the
  // register so that every immediate offset stays below 64K.
  constexpr int KB = 3 * HT_BYTES;
  uint32_t ka[8], va[4];
  {
    const uint32_t kbase = lq * 256 + (((lq & 15) ^ hh) << 4);           // natural, 16 granules per row
    const uint32_t vbase = lq * 128 + ((((lq >> 1) & 7) ^ hh) << 4);     // transposed, 8 granules per row
#pragma unroll
    for (int j = 0; j < 8; ++j) ka[j] = (kbase ^ (j << 5)) + KB;  // K buffers sit above the V buffers
#pragma unroll
    for (int j = 0; j < 4; ++j) va[j] = vbase ^ (j << 5);
  }

  // half tile ht: page j = ht / 2, keys 64 (ht % 2) .. + 63 of it
  auto ht_first = [&](int32_t ht) -> int64_t { return (int64_t)pw.page(ht >> 1) * TP + (ht & 1) * HT; };
  // Staging.  K (natural) and V (transposed) half tiles come from images that already have the byte
  // order of the LDS tiles, one 16 KiB image per half tile of the page list, so a half tile is copied
  // with direct global -> LDS loads: no staging registers, no LDS store instructions, and a whole
  // iteration of flight time.  The kernel waits for them itself before the barrier that publishes the
  // data.  Wave w moves bytes 2048 w .. + 2047 of each image.
  const unsigned char* const k_img_g = k_img + (size_t)g * img_len * 16384;
  const unsigned char* const vt_img_g = vt_img + (size_t)g * img_len * 16384;
  const uint32_t cp_off = 2048 * wave + 16 * lane;
  auto copy_tile = [&](const unsigned char* src, const uint32_t lds_dst) __attribute__((always_inline)) {
    copy_kib_to_lds<2>(src, cp_off, lds_dst + 2048 * wave);
  };
  // image index of half tile ht of the list: the list position itself, or (one list per query page) the
  // page's position in the KV head's union list, whose images are shared by all query pages
  auto img_ht = [&](int32_t ht) __attribute__((always_inline)) -> size_t {
    return (size_t)(p.qp ? 2 * pw.phys(ht >> 1) + (ht & 1) : ht) * 16384;
  };
  auto copy_k = [&](int32_t ht, const int buf) __attribute__((always_inline)) { copy_tile(k_img_g + img_ht(ht), KB + buf * HT_BYTES); };
  auto copy_v = [&](int32_t ht, const int buf) __attribute__((always_inline)) { copy_tile(vt_img_g + img_ht(ht), buf * HT_BYTES); };
  auto copies_landed = [&]() __attribute__((always_inline)) { wait_copies<0>(); };

  // ---- the software pipeline -------------------------------------------------------
  // A unit is 32 keys (half of a half tile).  One step of the pipeline runs three
  // mutually independent instruction streams, so matrix and vector instructions of one
  // wave overlap whatever the other wave of the SIMD is doing:
  //   matrix: O += V_u P_u (8 MFMA) interleaved with S_{u+2} = K_{u+2} Q^T (8 MFMA)
  //   vector: online softmax of S_{u+1} -> P_{u+1}, row sum, pending rescale factor
  //   LDS:    operand fragments, one batch of four ahead (the last batch of a step
  //           fetches the first batch of the next step)
  // The step is written as 16 slots of one MFMA + one fragment read + one slice of the
  // softmax; sched_barrier keeps the slots in source order.
  u32x4 fr[8];  // two batches of four fragments
  float t0 = 0.f, t1 = 0.f, t2 = 0.f, t3 = 0.f, t4 = 0.f, rs = 0.f, mc = 0.f, alpha_new = 1.f;

  // fragment e of batch b: e = 0, 2 -> K rows of k-steps 2b, 2b+1; e = 1, 3 -> V^T rows of dim block b.
  // ko / vo are compile-time byte offsets of the K unit and the V half tile in LDS, so every address
  // is a loop-invariant register plus an immediate
  auto frag = [&](const int ko, const int vo, int v, int b, int e) __attribute__((always_inline)) -> u32x4 {
    if ((e & 1) == 0) return *reinterpret_cast<const u32x4*>(smem + (ka[2 * b + (e >> 1)] + ko));
    return *reinterpret_cast<const u32x4*>(smem + (va[2 * v + (e >> 1)] + (vo + 4096 * b)));
  };
  // slice sl of the softmax of one unit: scores s (C layout: register x = key 8 (x / 4) + 4 hh + x % 4)
  // -> bf16 probabilities pr; rel = largest visible key index of this lane's row, less 4 hh
  auto sm_slice = [&](const int sl, f32x16& s, u32x4* pr, const int rel, const bool general) __attribute__((always_inline)) {
    if (sl == 0) {
      if (general) {
#pragma unroll
        for (int x = 0; x < 16; ++x)
          if (8 * (x >> 2) + (x & 3) > rel) s[x] = -INFINITY;
      }
      t0 = fmaxf(fmaxf(s[0], s[1]), s[2]);
      t1 = fmaxf(fmaxf(s[3], s[4]), s[5]);
    } else if (sl == 1) {
      t2 = fmaxf(fmaxf(s[6], s[7]), s[8]);
      t3 = fmaxf(fmaxf(s[9], s[10]), s[11]);
      t4 = fmaxf(fmaxf(s[12], s[13]), s[14]);
    } else if (sl == 2) {
      t0 = fmaxf(fmaxf(t0, t1), t2);
      t3 = fmaxf(fmaxf(t3, t4), s[15]);
      t0 = half_max(fmaxf(t0, t3));
    } else if (sl == 3) {
      const float m_new = fmaxf(m_run, t0);
      alpha_new = __builtin_amdgcn_exp2f((m_run - m_new) * c);
      m_run = m_new;
      mc = m_new * c;
      rs = 0.f;
    } else if (sl < 12) {
      const int x = 2 * (sl - 4);
      s[x] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[x], c, -mc));
      s[x + 1] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[x + 1], c, -mc));
    } else {
      const int q = sl - 12;
      const uint32_t w0 = pack2_bf16(s[4 * q + 0], s[4 * q + 1]);
      const uint32_t w1 = pack2_bf16(s[4 * q + 2], s[4 * q + 3]);
      rs = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w0), ones, rs, false);
      rs = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w1), ones, rs, false);
      pr[q >> 1][2 * (q & 1) + 0] = w0;
      pr[q >> 1][2 * (q & 1) + 1] = w1;
      if (sl == 15) {
        l_run = __builtin_fmaf(l_run, alpha_new, rs);
        alpha_pend = alpha_new;
      }
    }
  };
  // one pipeline step.  v = which half of the half tiles (K rows 32 v .., V token groups 2 v, 2 v + 1);
  // (ko, vo) = LDS offsets of this step's operands, (kn, vn) = those of the next step (which has v ^ 1)
  auto step = [&](const int v, const int ko, const int vo, const int kn, const int vn, f32x16& s_in, u32x4* p_out,
                  const u32x4* p_in, f32x16& s_out, const int rel, const bool general) __attribute__((always_inline)) {
    // rescale left pending by the previous softmax: O and l are multiplied only when some row's maximum moved
    if (__any(alpha_pend != 1.f)) {  // wave-uniform
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int x = 0; x < 16; ++x) of[db][x] *= alpha_pend;
    }
#pragma unroll
    for (int x = 0; x < 16; ++x) s_out[x] = 0.f;
#pragma unroll
    for (int sl = 0; sl < 16; ++sl) {
      const int b = sl >> 2, q = sl & 3;
      const int cur = 4 * (b & 1), nxt = 4 - cur;
      if (q == 0) {  // the whole next batch at once: one wait per batch instead of one per fragment
#pragma unroll
        for (int e = 0; e < 4; ++e) fr[nxt + e] = b < 3 ? frag(ko, vo, v, b + 1, e) : frag(kn, vn, v ^ 1, 0, e);
        __builtin_amdgcn_s_waitcnt(0xC47F);  // lgkmcnt(4): the batch fetched one batch ago has arrived
        __builtin_amdgcn_sched_barrier(0);   // keep the fetch ahead of this batch's matrix instructions
      }
      if (q == 0) s_out = mfma32(__builtin_bit_cast(bf16x8, fr[cur + 0]), qf[2 * b], s_out);
      if (q == 1) of[b] = mfma32(__builtin_bit_cast(bf16x8, fr[cur + 1]), __builtin_bit_cast(bf16x8, p_in[0]), of[b]);
      if (q == 2) s_out = mfma32(__builtin_bit_cast(bf16x8, fr[cur + 2]), qf[2 * b + 1], s_out);
      if (q == 3) of[b] = mfma32(__builtin_bit_cast(bf16x8, fr[cur + 3]), __builtin_bit_cast(bf16x8, p_in[1]), of[b]);
      sm_slice(sl, s_in, p_out, rel, general);
      __builtin_amdgcn_sched_barrier(0);
    }
    // keep this step's softmax in this step: without a use here the compiler sinks it into the
    // block of the next step, in front of that step's first matrix instruction
    asm volatile("" : "+v"(p_out[0]), "+v"(p_out[1]), "+v"(l_run), "+v"(alpha_pend));
  };
  // unpipelined S = K Q^T of one unit (prologue only)
  auto qk_plain = [&](f32x16& dst, const int ko) __attribute__((always_inline)) {
#pragma unroll
    for (int x = 0; x < 16; ++x) dst[x] = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      dst = mfma32(__builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(smem + (ka[j] + ko))), qf[j], dst);
  };
  auto rel_of = [&](int64_t first) -> int { return (int)(a_i - first) - 4 * hh; };

  // Half tiles [0, T_full) are seen in full by every row of the workgroup; steps whose
  // softmax unit lies in them need no mask.
  int32_t T_full = 0;
  {
    const int64_t a_blk_min = first_q + 32 * (int64_t)div_g(p, (uint32_t)rt.b_first);
    if (a_blk_min >= TP - 1) T_full = 2 * visible_len(p, lid, (a_blk_min - (TP - 1)) / TP, lane);
    if (T_full > T2) T_full = T2;
  }

  // prologue: K_0, K_1, K_2, V_0, V_1 into LDS; S_0, S_1, P_0
  if (T2 > 0) { copy_k(0, 0); copy_v(0, 0); }
  if (T2 > 1) { copy_k(1, 1); copy_v(1, 1); }
  if (T2 > 2) copy_k(2, 2);
  copies_landed();
  __syncthreads();
  if (T2 > 0 && r_valid) {
    qk_plain(sA, 0);
    qk_plain(sB, 8192);
    const int rel0 = rel_of(ht_first(0));
#pragma unroll
    for (int sl = 0; sl < 16; ++sl) sm_slice(sl, sA, pA, rel0, true);
#pragma unroll
    for (int q = 0; q < 4; ++q) fr[q] = frag(HT_BYTES, 0, 0, 0, q);
  }
  // iteration t (r = t mod 3): steps A (units 2t | 2t+1 | 2t+2) and B (2t+1 | 2t+2 | 2t+3); K_{t+1}
  // (buffer r+1) and V_t (buffer r) are read.  After the barrier between A and B the copies of K_{t+3}
  // (buffer r, whose K_t nobody reads any more) and V_{t+2} (buffer r+2, ex V_{t-1}) are issued; they
  // have to land before the next such barrier.  Three buffers each: a wave still in step B of the
  // previous iteration reads K_t and V_{t-1}.  The loops are unrolled by three so that r is a constant.
  auto iteration = [&](const int32_t t, const int r, const bool general) __attribute__((always_inline)) {
    const int kc = ((r + 1) % 3) * HT_BYTES, kw = ((r + 2) % 3) * HT_BYTES;
    const int vc = r * HT_BYTES, vw = ((r + 1) % 3) * HT_BYTES;
    pw.advance(p, lid, T, t >> 1, lane);
    int relA = 0, relB = 0;
    if (general) {
      relA = rel_of(ht_first(t) + 32);
      relB = t + 1 < T2 ? rel_of(ht_first(t + 1)) : -1;
    }
    // (a wave without a block of its own -- last row tile of a query page -- only moves data and
    // keeps the barriers, leaving the SIMD to its partner)
    if (r_valid) step(0, kc, vc, kc + 8192, vc, sB, pB, pA, sA, relA, general);
    copies_landed();
    __syncthreads();
    if (t + 3 < T2) copy_k(t + 3, r);
    if (t + 2 < T2) copy_v(t + 2, (r + 2) % 3);
    if (r_valid) step(1, kc + 8192, vc, kw, vw, sA, pA, pB, sB, relB, general);
  };
  {
    int32_t t = 0;
    for (; t + 3 < T_full; t += 3) {
      iteration(t, 0, false);
      iteration(t + 1, 1, false);
      iteration(t + 2, 2, false);
    }
    for (; t < T2; t += 3) {
      iteration(t, 0, true);
      if (t + 1 < T2) iteration(t + 1, 1, true);
      if (t + 2 < T2) iteration(t + 2, 2, true);
    }
  }
  // the last softmax (a fully masked unit) leaves alpha_pend = 1: nothing is pending here

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
  // (token strides: the direct copies of the backward kernels address the rows of a tile with a 32-bit lane offset)
  return is_bf16 && p.D == HD && p.P == TP && p.pool_tok_stride <= (1 << 20) && p.q_tok_stride <= (1 << 20);
}

size_t fwd_mfma_workspace_bytes(const Params& p, int32_t max_list_len) {
  return kv_image_bytes(p, max_list_len);
}

hipError_t launch_fwd_mfma(const Params& p, int32_t max_list_len, void* ws, hipStream_t st) {
  static DeviceOnce lds_once;
  if (hipError_t e = ensure_max_dynamic_lds(lds_once, (const void*)fwd_mfma_kernel, FW_LDS); e != hipSuccess) return e;
  const int tiles = row_tiles_per_head(p.C, p.G, p.m, p.qp);
  const int xcd_map = (p.Hkv <= 8 && 8 % p.Hkv == 0) ? 1 : 0;
  unsigned blocks;
  if (xcd_map) {
    const int per = 8 / p.Hkv;
    blocks = 8u * (unsigned)((tiles + per - 1) / per);
  } else {
    blocks = (unsigned)tiles * p.Hkv;
  }
  hipError_t e = launch_kv_layout(p, max_list_len, ws, st);
  if (e != hipSuccess) return e;
  const unsigned char* k_img = (const unsigned char*)ws;
  const unsigned char* vt_img = k_img + kv_image_bytes(p, max_list_len) / 2;
  { ProfScope prof_("attn_fwd_mfma", st); fwd_mfma_kernel<<<dim3(blocks), dim3(FW_THREADS), FW_LDS, st>>>(p, tiles, xcd_map, k_img, vt_img, 2 * max_list_len); }
  return hipGetLastError();
}

}  // namespace oomb
