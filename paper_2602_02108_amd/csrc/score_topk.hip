// Page scoring and top-k page selection (paper Sec. 4.2): the mean of each key
// page is scored against the mean-pooled chunk query of its KV head and the
// top-K past pages are kept, plus the chunk's own pages.
//
// The fp32 operation order is fixed so that scores are reproducible bit for bit:
//   token sums left to right; qbar sums query pages (outer) then heads (inner);
//   dot product as a stride-halving tree over d.  No fused multiply-add.
// The page-mean kernel is HBM-bound: it streams every past key once.
#include <mutex>

#include "common.h"
#include "launch.h"
#include "rowsum.h"

#pragma clang fp contract(off)

namespace oomb {

// Step S1a: A[h][tau][d] = sum over the P tokens of query page tau of Q.  Every (head, query page, lane's
// d) is one sequential chain of P additions: the chains are all the parallelism there is, so they are spread
// one wave per workgroup over as many compute units as possible, each lane with 32 loads in flight.
constexpr int QPOOL_THREADS = 64;
template <typename T, int D>
__global__ __launch_bounds__(QPOOL_THREADS) void qpool_partial_kernel(Params p, float* __restrict__ A) {
  constexpr int VEC = Vec16<T>::N, LPR = D / VEC, UPB = QPOOL_THREADS / LPR;
  const int unit = blockIdx.x * UPB + threadIdx.x / LPR;
  const int lr = threadIdx.x % LPR;
  if (unit >= p.Hq * p.m) return;
  const int h = unit / p.m, tau = unit % p.m;
  const T* base = (const T*)p.q + (int64_t)tau * p.P * p.q_tok_stride + (int64_t)h * p.q_head_stride + lr * VEC;
  float acc[VEC];
  seq_row_sum<T, 32>(base, p.q_tok_stride, p.P, acc);
  float* out = A + ((int64_t)h * p.m + tau) * D + lr * VEC;
#pragma unroll
  for (int v = 0; v < VEC; ++v) out[v] = acc[v];
}

// Step S1b: qbar[g][d] = (sum over tau (outer), heads of g (inner) of A) * r.  One workgroup per KV head.  The
// sum of a (g, d) is one sequential chain over the m G terms k = tau * G + (h - g G); the terms are brought
// into LDS by all threads at once (rows of D floats, FINAL_ROWS at a time), then thread d walks its chain.
constexpr int FINAL_THREADS = 1024;
constexpr int FINAL_LDS_FLOATS = 32768;  // 128 KiB
__global__ __launch_bounds__(FINAL_THREADS) void qpool_final_kernel(Params p, const float* __restrict__ A,
                                                                    float* __restrict__ qbar, float r) {
  extern __shared__ float rows[];  // [rows per pass][D]
  const int g = blockIdx.x, tid = threadIdx.x, D = p.D;
  const int dshift = D == 128 ? 7 : 6;  // D is 64 or 128
  const int n = p.m * p.G;
  const int per_pass = FINAL_LDS_FLOATS >> dshift;
  float acc = 0.0f;
  for (int k0 = 0; k0 < n; k0 += per_pass) {
    const int cnt = n - k0 < per_pass ? n - k0 : per_pass;
    // (eight independent loads per thread in flight)
    const int total = cnt << dshift;
    for (int e0 = tid; e0 < total; e0 += 8 * FINAL_THREADS) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int e = e0 + u * FINAL_THREADS;
        const int k = k0 + (e >> dshift), d = e & (D - 1);
        const int tau = (int)div_g(p, (uint32_t)k), h = g * p.G + (k - tau * p.G);
        v[u] = e < total ? A[((int64_t)h * p.m + tau) * D + d] : 0.0f;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (e0 + u * FINAL_THREADS < total) rows[e0 + u * FINAL_THREADS] = v[u];
    }
    __syncthreads();
    if (tid < D) {
      // the reads are independent and issued 16 at a time; the additions stay in order
      int k = 0;
      for (; k + 16 <= cnt; k += 16) {
        float v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = rows[((k + u) << dshift) + tid];
#pragma unroll
        for (int u = 0; u < 16; ++u) acc = __fadd_rn(acc, v[u]);
      }
      for (; k < cnt; ++k) acc = __fadd_rn(acc, rows[(k << dshift) + tid]);
    }
    __syncthreads();
  }
  if (tid < D) qbar[g * D + tid] = __fmul_rn(acc, r);
}

// Steps S2 + S3: one group of LPR lanes walks one (KV head, logical page) tile
// of the K pool token by token; a wave covers 64 / LPR pages at once.
template <typename T, int D>
__global__ __launch_bounds__(256) void page_score_kernel(Params p, const float* __restrict__ qbar,
                                                         float* __restrict__ scores, float inv_p) {
  constexpr int VEC = Vec16<T>::N, LPR = D / VEC, PPB = 256 / LPR;
  const int g = blockIdx.y;
  const int lr = threadIdx.x % LPR;
  const int64_t l = (int64_t)blockIdx.x * PPB + threadIdx.x / LPR;
  const bool active = l < p.n_past;
  const int64_t lc = active ? l : 0;
  const T* base = (const T*)p.k_pool + (int64_t)p.page_table[lc] * p.pool_page_stride +
                  (int64_t)g * p.pool_head_stride + lr * VEC;
  float x[VEC];
  seq_row_sum<T, 16, true>(base, p.pool_tok_stride, p.P, x);
  const float* qb = qbar + g * D + lr * VEC;
#pragma unroll
  for (int v = 0; v < VEC; ++v) x[v] = __fmul_rn(qb[v], __fmul_rn(x[v], inv_p));
  // tree over d: strides D/2 .. VEC cross lanes, then VEC/2 .. 1 inside the lane
#pragma unroll
  for (int s = D / 2; s >= VEC; s >>= 1) {
#pragma unroll
    for (int v = 0; v < VEC; ++v) x[v] = __fadd_rn(x[v], __shfl_xor(x[v], s / VEC, 64));
  }
#pragma unroll
  for (int s = VEC / 2; s >= 1; s >>= 1) {
#pragma unroll
    for (int v = 0; v < VEC; ++v)
      if (v < s) x[v] = __fadd_rn(x[v], x[v + s]);
  }
  if (active && lr == 0) scores[(int64_t)g * p.n_past + l] = x[0];
}

// Order-preserving map float -> uint32 (larger float = larger key); -0 maps with +0.
__device__ __forceinline__ uint32_t order_key(float s) {
  uint32_t b = __float_as_uint(s);
  if ((b << 1) == 0u) b = 0u;
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

constexpr int SELECT_THREADS = 1024;

// block-wide sum of a 64-bit value (used for three 21-bit counters packed in one word)
__device__ __forceinline__ unsigned long long block_sum64(unsigned long long v, unsigned long long* smem /*[16]*/) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();  // protects smem reuse across calls
  if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
  __syncthreads();
  unsigned long long tot = 0;
#pragma unroll
  for (int w = 0; w < SELECT_THREADS / 64; ++w) tot += smem[w];
  return tot;
}

// Step S4.  One workgroup per list: per KV head, or (per_qp) per KV head and query page tau =
// blockIdx.x % m, whose list ends with the tau + 1 local pages its rows can see.  The k-th largest
// key is found by bisection over its 32 bits (count of keys >= candidate), then the list is
// emitted in ascending logical id: all keys above the threshold, the lowest-id
// keys equal to it, and the local pages.
__global__ __launch_bounds__(SELECT_THREADS) void topk_select_kernel(
    const float* __restrict__ scores, int64_t n_past, int32_t m, int32_t top_k,
    int32_t* __restrict__ sel, int32_t* __restrict__ sel_count, int32_t lds_cap, int32_t per_qp) {
  extern __shared__ uint32_t keys[];  // first min(n_past, lds_cap) keys cached
  __shared__ unsigned long long red[SELECT_THREADS / 64];
  const int g = blockIdx.x, tid = threadIdx.x;
  const int32_t n_loc = per_qp ? (int32_t)(blockIdx.x % m) + 1 : m;
  const float* sc = scores + (int64_t)g * n_past;
  const int32_t stride = top_k + m;
  int32_t* out = sel + (int64_t)g * stride;
  const int32_t k_eff = (int32_t)(top_k < n_past ? top_k : n_past);
  const int64_t cached = n_past < lds_cap ? n_past : lds_cap;

  for (int64_t l = tid; l < cached; l += SELECT_THREADS) keys[l] = order_key(sc[l]);
  __syncthreads();
  auto key_at = [&](int64_t l) -> uint32_t { return l < cached ? keys[l] : order_key(sc[l]); };

  // T = the k_eff-th largest key = the largest T with #(key >= T) >= k_eff, found two bits at
  // a time: the counts for the three candidates T | (1..3 << b) travel in one 64-bit sum
  // (21 bits each; n_past <= 2^20).
  uint32_t T = 0;
  int take_eq = 0;
  if (k_eff > 0) {
    for (int b = 30; b >= 0; b -= 2) {
      const uint32_t c1 = T | (1u << b), c2 = T | (2u << b), c3 = T | (3u << b);
      unsigned long long c = 0;
      for (int64_t l = tid; l < n_past; l += SELECT_THREADS) {
        const uint32_t k = key_at(l);
        c += (unsigned long long)(k >= c1) | ((unsigned long long)(k >= c2) << 21) | ((unsigned long long)(k >= c3) << 42);
      }
      const unsigned long long tot = block_sum64(c, red);
      const int n1 = (int)(tot & 0x1fffff), n2 = (int)((tot >> 21) & 0x1fffff), n3 = (int)((tot >> 42) & 0x1fffff);
      if (n3 >= k_eff) T = c3;
      else if (n2 >= k_eff) T = c2;
      else if (n1 >= k_eff) T = c1;
    }
    unsigned long long c = 0;
    for (int64_t l = tid; l < n_past; l += SELECT_THREADS) c += key_at(l) > T;
    take_eq = k_eff - (int)block_sum64(c, red);  // how many keys equal to T are kept (lowest ids)
  }

  // ordered emission: thread t owns the contiguous id range [t*per, (t+1)*per)
  const int64_t per = (n_past + SELECT_THREADS - 1) / SELECT_THREADS;
  const int64_t lo = (int64_t)tid * per, hi = (lo + per < n_past) ? lo + per : n_past;
  int n_eq = 0, n_gt = 0;
  if (k_eff > 0)
    for (int64_t l = lo; l < hi; ++l) {
      const uint32_t k = key_at(l);
      n_eq += k == T;
      n_gt += k > T;
    }
  // exclusive scans of (n_eq, n_gt) over threads, packed in one 64-bit add
  unsigned long long v = ((unsigned long long)(uint32_t)n_eq << 32) | (uint32_t)n_gt;
  unsigned long long incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    unsigned long long nb = __shfl_up(incl, o, 64);
    if ((tid & 63) >= o) incl += nb;
  }
  __shared__ unsigned long long wave_tot[SELECT_THREADS / 64];
  if ((tid & 63) == 63) wave_tot[tid >> 6] = incl;
  __syncthreads();
  unsigned long long base = 0;
  for (int w = 0; w < (tid >> 6); ++w) base += wave_tot[w];
  const unsigned long long excl = base + incl - v;
  int eq_before = (int)(excl >> 32);
  int gt_before = (int)(excl & 0xffffffffu);
  if (k_eff > 0) {
    // position = kept keys with lower id = gt_before + min(eq_before, take_eq)
    int pos = gt_before + (eq_before < take_eq ? eq_before : take_eq);
    for (int64_t l = lo; l < hi; ++l) {
      const uint32_t k = key_at(l);
      if (k > T) {
        out[pos++] = (int32_t)l;
      } else if (k == T) {
        if (eq_before < take_eq) out[pos++] = (int32_t)l;
        ++eq_before;
      }
    }
  }
  for (int32_t j = tid; j < n_loc; j += SELECT_THREADS) out[k_eff + j] = (int32_t)(n_past + j);
  for (int32_t j = k_eff + n_loc + tid; j < stride; j += SELECT_THREADS) out[j] = -1;
  if (tid == 0) sel_count[g] = k_eff + n_loc;
}

// Step S4 for lists of at most PER * SELECT_THREADS candidates: the same selection with the keys held in
// registers.  Thread t owns the PER consecutive ids from t PER on, so nothing is re-read from memory.  The
// k_eff-th largest key is found by a radix select, eight bits per pass from the top: every wave counts the
// byte of its keys that still match the prefix into a histogram of its own in LDS (integer additions: the
// order does not matter), 256 threads add the 16 histograms and scan them from the top, and the bin where
// the count crosses what is still wanted extends the prefix.  Four passes, three barriers each; the ordered
// emission needs only the exclusive scan over threads.
template <int PER>
__global__ __launch_bounds__(SELECT_THREADS) void topk_select_reg_kernel(
    const float* __restrict__ scores, int64_t n_past, int32_t m, int32_t top_k,
    int32_t* __restrict__ sel, int32_t* __restrict__ sel_count, int32_t per_qp) {
  constexpr int WAVES = SELECT_THREADS / 64;
  __shared__ uint32_t hist[2][WAVES][256];
  __shared__ uint32_t scan_tot[4];
  __shared__ uint32_t picked[2];  // {bin, how many keys of that bin are still wanted}
  __shared__ unsigned long long wave_tot[WAVES];
  const int g = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t n_loc = per_qp ? (int32_t)(blockIdx.x % m) + 1 : m;
  const float* sc = scores + (int64_t)g * n_past;
  const int32_t stride = top_k + m;
  int32_t* out = sel + (int64_t)g * stride;
  const int32_t k_eff = (int32_t)(top_k < n_past ? top_k : n_past);
  const int32_t np = (int32_t)n_past;

  for (int e = tid; e < WAVES * 256; e += SELECT_THREADS) (&hist[0][0][0])[e] = 0u;
  const int32_t lo = tid * PER;
  uint32_t key[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) key[i] = lo + i < np ? order_key(sc[lo + i]) : 0u;
  __syncthreads();

  uint32_t T = 0;
  int take_eq = 0;
  if (k_eff > 0) {
    uint32_t want = (uint32_t)k_eff;  // keys still wanted among those that match the prefix
#pragma unroll 1
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass, cur = pass & 1;
      // the other histogram set is free: clear it for the next pass
      for (int e = tid; e < WAVES * 256; e += SELECT_THREADS) (&hist[cur ^ 1][0][0])[e] = 0u;
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const bool match = lo + i < np && (pass == 0 || (key[i] >> (shift + 8)) == (T >> (shift + 8)));
        if (match) atomicAdd(&hist[cur][wave][(key[i] >> shift) & 255u], 1u);
      }
      __syncthreads();
      // thread t < 256 takes bin 255 - t: an inclusive scan over t is the count of keys in bins >= its own
      uint32_t v = 0, inc = 0;
      if (tid < 256) {
#pragma unroll
        for (int w = 0; w < WAVES; ++w) v += hist[cur][w][255 - tid];
        inc = v;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const uint32_t nb = __shfl_up(inc, o, 64);
          if (lane >= o) inc += nb;
        }
        if (lane == 63) scan_tot[wave] = inc;
      }
      __syncthreads();
      if (tid < 256) {
        for (int w = 0; w < wave; ++w) inc += scan_tot[w];
        const uint32_t above = inc - v;  // keys in higher bins
        if (inc >= want && above < want) {
          picked[0] = 255u - (uint32_t)tid;
          picked[1] = want - above;
        }
      }
      __syncthreads();
      T |= picked[0] << shift;
      want = picked[1];
    }
    take_eq = (int)want;  // how many keys equal to T are kept (lowest ids)
  }

  int n_eq = 0, n_gt = 0;
  if (k_eff > 0) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const bool valid = lo + i < np;
      n_eq += valid && key[i] == T;
      n_gt += valid && key[i] > T;
    }
  }
  // exclusive scans of (n_eq, n_gt) over threads, packed in one 64-bit add
  const unsigned long long v = ((unsigned long long)(uint32_t)n_eq << 32) | (uint32_t)n_gt;
  unsigned long long incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned long long nb = __shfl_up(incl, o, 64);
    if (lane >= o) incl += nb;
  }
  if (lane == 63) wave_tot[tid >> 6] = incl;
  __syncthreads();
  unsigned long long base = 0;
  for (int w = 0; w < (tid >> 6); ++w) base += wave_tot[w];
  const unsigned long long excl = base + incl - v;
  int eq_before = (int)(excl >> 32);
  const int gt_before = (int)(excl & 0xffffffffu);
  if (k_eff > 0) {
    // position = kept keys with lower id = gt_before + min(eq_before, take_eq)
    int pos = gt_before + (eq_before < take_eq ? eq_before : take_eq);
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      if (lo + i < np) {
        if (key[i] > T) {
          out[pos++] = lo + i;
        } else if (key[i] == T) {
          if (eq_before < take_eq) out[pos++] = lo + i;
          ++eq_before;
        }
      }
    }
  }
  for (int32_t j = tid; j < n_loc; j += SELECT_THREADS) out[k_eff + j] = (int32_t)(n_past + j);
  for (int32_t j = k_eff + n_loc + tid; j < stride; j += SELECT_THREADS) out[j] = -1;
  if (tid == 0) sel_count[g] = k_eff + n_loc;
}

static hipError_t launch_topk_select(const Params& p, const float* scores, int32_t top_k, int32_t* sel, int32_t* sel_count,
                                     int per_qp, hipStream_t st) {
  const dim3 grid((unsigned)(per_qp ? p.Hkv * p.m : p.Hkv)), block(SELECT_THREADS);
  const int64_t per = (p.n_past + SELECT_THREADS - 1) / SELECT_THREADS;
  if (per <= 32) {  // the keys of a list fit the registers of one workgroup
    ProfScope prof_("topk_select", st);
#define OOMB_TOPK_REG(PER) topk_select_reg_kernel<PER><<<grid, block, 0, st>>>(scores, p.n_past, p.m, top_k, sel, sel_count, per_qp)
    if (per <= 2) OOMB_TOPK_REG(2);
    else if (per <= 4) OOMB_TOPK_REG(4);
    else if (per <= 8) OOMB_TOPK_REG(8);
    else if (per <= 12) OOMB_TOPK_REG(12);
    else if (per <= 16) OOMB_TOPK_REG(16);
    else if (per <= 24) OOMB_TOPK_REG(24);
    else OOMB_TOPK_REG(32);
#undef OOMB_TOPK_REG
    return hipGetLastError();
  }
  constexpr int WANT = 144 * 1024;
  static DeviceOnce lds_once;
  if (hipError_t e = ensure_max_dynamic_lds(lds_once, (const void*)topk_select_kernel, WANT); e != hipSuccess) return e;
  const int64_t cap = WANT / 4;
  const int64_t cached = p.n_past < cap ? p.n_past : cap;
  ProfScope prof_("topk_select", st);
  topk_select_kernel<<<grid, block, (size_t)cached * 4, st>>>(
      scores, p.n_past, p.m, top_k, sel, sel_count, (int32_t)cap, per_qp);
  return hipGetLastError();
}

// kbar_cache != nullptr: the page means come from the cache instead of the keys
template <typename T, int D>
static hipError_t launch_scoring(const Params& p, float* A, float* qbar, float* scores, const float* kbar_cache, hipStream_t st) {
  constexpr int VEC = Vec16<T>::N, LPR = D / VEC, PER_BLOCK = 256 / LPR;
  const int units = p.Hq * p.m;
  constexpr int UPB = QPOOL_THREADS / LPR;
  { ProfScope prof_("qpool_partial", st); qpool_partial_kernel<T, D><<<dim3((units + UPB - 1) / UPB), dim3(QPOOL_THREADS), 0, st>>>(p, A); }
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  const float r = 1.0f / (float)((int64_t)p.C * p.G);
  {
    static DeviceOnce lds_once;
    if (hipError_t e = ensure_max_dynamic_lds(lds_once, (const void*)qpool_final_kernel, FINAL_LDS_FLOATS * 4); e != hipSuccess) return e;
    ProfScope prof_("qpool_final", st);
    qpool_final_kernel<<<dim3(p.Hkv), dim3(FINAL_THREADS), FINAL_LDS_FLOATS * 4, st>>>(p, A, qbar, r);
  }
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  if (kbar_cache) return launch_page_score_cached(p, qbar, kbar_cache, scores, st);
  if (p.n_past > 0) {
    const float inv_p = 1.0f / (float)p.P;
    dim3 grid((unsigned)((p.n_past + PER_BLOCK - 1) / PER_BLOCK), p.Hkv);
    { ProfScope prof_("page_score", st); page_score_kernel<T, D><<<grid, dim3(256), 0, st>>>(p, qbar, scores, inv_p); }
    return hipGetLastError();
  }
  return hipSuccess;
}

size_t score_workspace_bytes(const Params& p) {
  size_t a = (size_t)p.Hq * p.m * p.D * sizeof(float);
  size_t qb = (size_t)p.Hkv * p.D * sizeof(float);
  size_t sc = (size_t)p.Hkv * (size_t)(p.n_past > 0 ? p.n_past : 1) * sizeof(float);
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  return up(a) + up(qb) + up(sc);
}

// Returns hipSuccess or the launch error.  dtype_is_bf16 picks the element type.
hipError_t launch_score_topk(const Params& p, bool is_bf16, int32_t top_k, int32_t* sel,
                             int32_t* sel_count, float* scores_out, void* ws, const float* kbar_cache, hipStream_t st) {
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  char* w = (char*)ws;
  float* A = (float*)w;
  w += up((size_t)p.Hq * p.m * p.D * sizeof(float));
  float* qbar = (float*)w;
  w += up((size_t)p.Hkv * p.D * sizeof(float));
  float* scores = scores_out ? scores_out : (float*)w;

  hipError_t e;
  if (is_bf16) {
    e = p.D == 128 ? launch_scoring<bf16_t, 128>(p, A, qbar, scores, kbar_cache, st)
                   : launch_scoring<bf16_t, 64>(p, A, qbar, scores, kbar_cache, st);
  } else {
    e = p.D == 128 ? launch_scoring<float, 128>(p, A, qbar, scores, kbar_cache, st)
                   : launch_scoring<float, 64>(p, A, qbar, scores, kbar_cache, st);
  }
  if (e != hipSuccess) return e;
  return launch_topk_select(p, scores, top_k, sel, sel_count, 0, st);
}

// Built-in scratch memory of oomb_page_score_topk_noalloc: the scoring workspace (query-page sums, pooled
// queries, scores) for callers that cannot hand one over.  Every device the library runs on holds its own
// copy of the array until the process ends.  In host code the array's name is only a stand-in; the address
// on the current device comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[OOMB_NOALLOC_SCRATCH_BYTES];

hipError_t score_scratch_ptr(void** out) {
  constexpr int MAX_DEVICES = 64;
  static std::mutex mu;
  static void* ptrs[MAX_DEVICES] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(mu);
  if (!ptrs[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    ptrs[dev] = ptr;
  }
  *out = ptrs[dev];
  return hipSuccess;
}

// votes [Hkv][m][n_past] -> one list per (KV head, query page), sel [Hkv][m][top_k + m]
hipError_t launch_topk_select_qp(const Params& p, const float* votes, int32_t top_k, int32_t* sel, int32_t* sel_count,
                                 hipStream_t st) {
  return launch_topk_select(p, votes, top_k, sel, sel_count, 1, st);
}

}  // namespace oomb
