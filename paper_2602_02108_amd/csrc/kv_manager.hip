// Paged-manager steps either side of the attention path (paper Sec. 4.1: the KV cache grows chunk
// by chunk in pages; Sec. 4.2: page means represent the pages, local-attention layers retrieve the
// most recent pages):
//   kv_append          the chunk's K / V -> its m local pages in the pools
//   page_means         mean of each page of a range -> cache [logical page][KV head][D] (fp32)
//   page_score_cached  scores from the cached means instead of streaming the keys
//   local_page_list    the page list of a local-attention layer
// The means and scores use the fixed fp32 operation order of the streaming scorer
// (score_topk.hip), so both paths give the same bits.
#include "common.h"
#include "launch.h"
#include "rowsum.h"

#pragma clang fp contract(off)

namespace oomb {

// chunk K / V [C][Hkv][D] (contiguous) -> pool pages page_table[n_past + i / P]; 16 bytes per thread
template <int ES>
__global__ __launch_bounds__(256) void kv_append_kernel(Params p, const unsigned char* __restrict__ kc,
                                                        const unsigned char* __restrict__ vc,
                                                        unsigned char* __restrict__ k_pool,
                                                        unsigned char* __restrict__ v_pool) {
  const int gpr = p.D * ES / 16;  // 16-byte granules per (token, head) row
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = (int64_t)p.C * p.Hkv * gpr;
  if (idx >= total) return;
  const int c = (int)(idx % gpr);
  const int64_t row = idx / gpr;
  const int g = (int)(row % p.Hkv), i = (int)(row / p.Hkv);
  const int64_t src = (row * p.D) * ES + c * 16;
  const int64_t dst = ((int64_t)p.page_table[p.n_past + i / p.P] * p.pool_page_stride + (int64_t)g * p.pool_head_stride +
                       (int64_t)(i % p.P) * p.pool_tok_stride) * ES + c * 16;
  *reinterpret_cast<uint4*>(k_pool + dst) = *reinterpret_cast<const uint4*>(kc + src);
  *reinterpret_cast<uint4*>(v_pool + dst) = *reinterpret_cast<const uint4*>(vc + src);
}

// mean of logical pages [first, first + count): one thread per (page, head, d); tokens left to right
template <typename T>
__global__ __launch_bounds__(256) void page_means_kernel(Params p, int64_t first, int64_t count, float inv_p,
                                                         float* __restrict__ cache) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= count * p.Hkv * p.D) return;
  const int d = (int)(idx % p.D);
  const int g = (int)((idx / p.D) % p.Hkv);
  const int64_t l = first + idx / ((int64_t)p.D * p.Hkv);
  const T* base = (const T*)p.k_pool + (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride + d;
  float acc = 0.0f;
  for (int t = 0; t < p.P; ++t) acc = __fadd_rn(acc, Elem<T>::load(base + (int64_t)t * p.pool_tok_stride));
  cache[((int64_t)l * p.Hkv + g) * p.D + d] = __fmul_rn(acc, inv_p);
}

// The same means for D = 64 / 128 with 16-byte loads: a group of LPR lanes walks one (page, KV head)
// tile token by token (same addition order, same bits); this is the kernel that streams a whole
// history when the means are not cached.
template <typename T, int D>
__global__ __launch_bounds__(256) void page_means_vec_kernel(Params p, int64_t first, int64_t count, float inv_p,
                                                             float* __restrict__ cache) {
  constexpr int VEC = Vec16<T>::N, LPR = D / VEC, PPB = 256 / LPR;
  const int g = blockIdx.y;
  const int lr = threadIdx.x % LPR;
  const int64_t k = (int64_t)blockIdx.x * PPB + threadIdx.x / LPR;
  if (k >= count) return;
  const int64_t l = first + k;
  const T* base = (const T*)p.k_pool + (int64_t)p.page_table[l] * p.pool_page_stride +
                  (int64_t)g * p.pool_head_stride + lr * VEC;
  float x[VEC];
  seq_row_sum<T, 8, true>(base, p.pool_tok_stride, p.P, x);
  float* out = cache + ((int64_t)l * p.Hkv + g) * D + lr * VEC;
#pragma unroll
  for (int v = 0; v < VEC; ++v) out[v] = __fmul_rn(x[v], inv_p);
}

// score[g][l] = tree sum over d of qbar[g][d] * cache[l][g][d] (stride-halving tree, strides D/2 .. 1):
// a group of D / 4 lanes per (head, page), four floats per lane
template <int D>
__global__ __launch_bounds__(256) void page_score_cached_kernel(Params p, const float* __restrict__ qbar,
                                                                const float* __restrict__ cache,
                                                                float* __restrict__ scores) {
  constexpr int VEC = 4, LPR = D / VEC, PPB = 256 / LPR;
  const int g = blockIdx.y;
  const int lr = threadIdx.x % LPR;
  const int64_t l = (int64_t)blockIdx.x * PPB + threadIdx.x / LPR;
  const bool active = l < p.n_past;
  const int64_t lc = active ? l : 0;
  const float4 kb = *reinterpret_cast<const float4*>(cache + ((int64_t)lc * p.Hkv + g) * D + lr * VEC);
  const float4 qb = *reinterpret_cast<const float4*>(qbar + g * D + lr * VEC);
  float x[VEC] = {__fmul_rn(qb.x, kb.x), __fmul_rn(qb.y, kb.y), __fmul_rn(qb.z, kb.z), __fmul_rn(qb.w, kb.w)};
#pragma unroll
  for (int s = D / 2; s >= VEC; s >>= 1) {
#pragma unroll
    for (int v = 0; v < VEC; ++v) x[v] = __fadd_rn(x[v], __shfl_xor(x[v], s / VEC, 64));
  }
  x[0] = __fadd_rn(x[0], x[2]);
  x[1] = __fadd_rn(x[1], x[3]);
  x[0] = __fadd_rn(x[0], x[1]);
  if (active && lr == 0) scores[(int64_t)g * p.n_past + l] = x[0];
}

__global__ void local_page_list_kernel(int64_t n_past, int64_t n, int32_t window, int32_t stride,
                                       int32_t* __restrict__ sel, int32_t* __restrict__ sel_count) {
  const int g = blockIdx.x;
  const int64_t w = window < n_past ? window : n_past;
  const int32_t cnt = (int32_t)(w + (n - n_past));
  for (int32_t j = threadIdx.x; j < stride; j += blockDim.x)
    sel[(int64_t)g * stride + j] = j < cnt ? (int32_t)(n_past - w + j) : -1;
  if (threadIdx.x == 0) sel_count[g] = cnt;
}

hipError_t launch_kv_append(const Params& p, bool is_bf16, const void* kc, const void* vc, void* k_pool, void* v_pool,
                            float* cache, hipStream_t st) {
  const int es = is_bf16 ? 2 : 4;
  const int64_t total = (int64_t)p.C * p.Hkv * (p.D * es / 16);
  {
    ProfScope prof_("kv_append", st);
    if (is_bf16)
      kv_append_kernel<2><<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(
          p, (const unsigned char*)kc, (const unsigned char*)vc, (unsigned char*)k_pool, (unsigned char*)v_pool);
    else
      kv_append_kernel<4><<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(
          p, (const unsigned char*)kc, (const unsigned char*)vc, (unsigned char*)k_pool, (unsigned char*)v_pool);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !cache) return e;
  const int64_t work = (int64_t)p.m * p.Hkv * p.D;
  const float inv_p = 1.0f / (float)p.P;
  ProfScope prof_("page_means", st);
  if (is_bf16) page_means_kernel<bf16_t><<<dim3((unsigned)((work + 255) / 256)), dim3(256), 0, st>>>(p, p.n_past, p.m, inv_p, cache);
  else page_means_kernel<float><<<dim3((unsigned)((work + 255) / 256)), dim3(256), 0, st>>>(p, p.n_past, p.m, inv_p, cache);
  return hipGetLastError();
}

hipError_t launch_page_means(const Params& p, bool is_bf16, int64_t first, int64_t count, float* cache, hipStream_t st) {
  if (count <= 0) return hipSuccess;
  const int64_t work = count * p.Hkv * p.D;
  const float inv_p = 1.0f / (float)p.P;
  ProfScope prof_("page_means", st);
  if (p.D == 128 || p.D == 64) {
    const int lpr = is_bf16 ? p.D / 8 : p.D / 4, ppb = 256 / lpr;
    dim3 grid((unsigned)((count + ppb - 1) / ppb), (unsigned)p.Hkv);
    if (is_bf16 && p.D == 128) page_means_vec_kernel<bf16_t, 128><<<grid, dim3(256), 0, st>>>(p, first, count, inv_p, cache);
    else if (is_bf16) page_means_vec_kernel<bf16_t, 64><<<grid, dim3(256), 0, st>>>(p, first, count, inv_p, cache);
    else if (p.D == 128) page_means_vec_kernel<float, 128><<<grid, dim3(256), 0, st>>>(p, first, count, inv_p, cache);
    else page_means_vec_kernel<float, 64><<<grid, dim3(256), 0, st>>>(p, first, count, inv_p, cache);
    return hipGetLastError();
  }
  if (is_bf16) page_means_kernel<bf16_t><<<dim3((unsigned)((work + 255) / 256)), dim3(256), 0, st>>>(p, first, count, inv_p, cache);
  else page_means_kernel<float><<<dim3((unsigned)((work + 255) / 256)), dim3(256), 0, st>>>(p, first, count, inv_p, cache);
  return hipGetLastError();
}

hipError_t launch_page_score_cached(const Params& p, const float* qbar, const float* cache, float* scores, hipStream_t st) {
  if (p.n_past <= 0) return hipSuccess;
  ProfScope prof_("page_score_cached", st);
  if (p.D == 128) {
    dim3 grid((unsigned)((p.n_past + 7) / 8), p.Hkv);
    page_score_cached_kernel<128><<<grid, dim3(256), 0, st>>>(p, qbar, cache, scores);
  } else {
    dim3 grid((unsigned)((p.n_past + 15) / 16), p.Hkv);
    page_score_cached_kernel<64><<<grid, dim3(256), 0, st>>>(p, qbar, cache, scores);
  }
  return hipGetLastError();
}

hipError_t launch_local_page_list(const Params& p, int32_t window, int32_t* sel, int32_t* sel_count, hipStream_t st) {
  ProfScope prof_("local_page_list", st);
  local_page_list_kernel<<<dim3(p.Hkv), dim3(256), 0, st>>>(p.n_past, p.n, window, window + p.m, sel, sel_count);
  return hipGetLastError();
}

}  // namespace oomb
