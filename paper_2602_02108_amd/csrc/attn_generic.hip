// Shape-generic paged attention kernels with fp32 arithmetic (no MFMA).  They
// serve fp32 tensors and the (D, P) combinations the MFMA kernels do not cover.
// One wave per query row (forward, dQ) or per owned key token (dK/dV), so the
// dK/dV pool is updated without atomics.  Forward: Sec. 4.1 operator; backward:
// Sec. 3 Eq. 3 accumulation into the paged gradient pool.
#include "common.h"
#include "launch.h"

namespace oomb {

constexpr int GEN_WAVES = 4;     // waves per workgroup
constexpr int GEN_MAX_D = 128;
constexpr int GEN_MAX_P = 128;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Delta[h][i] = <dO[i,h,:], O[i,h,:]>.  One wave per row.
template <typename T>
__global__ __launch_bounds__(256) void delta_kernel(Params p) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= (int64_t)p.C * p.Hq) return;
  const int i = (int)(row / p.Hq), h = (int)(row % p.Hq);
  const T* a = (const T*)p.d_o + (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride;
  const T* b = (const T*)p.o + (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride;
  float acc = 0.f;
  for (int d = lane; d < p.D; d += 64) acc += Elem<T>::load(a + d) * Elem<T>::load(b + d);
  acc = wave_sum(acc);
  if (lane == 0) p.delta[(int64_t)h * p.C + i] = acc;
}

template <typename T>
__global__ __launch_bounds__(64 * GEN_WAVES) void fwd_generic_kernel(Params p) {
  __shared__ float qs[GEN_WAVES][GEN_MAX_D];
  __shared__ float pb[GEN_WAVES][GEN_MAX_P];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * GEN_WAVES + w;
  if (row >= (int64_t)p.C * p.Hq) return;
  const int i = (int)(row / p.Hq), h = (int)(row % p.Hq), g = h / p.G;
  const int64_t a_i = p.N - p.C + i;
  const int D = p.D, P = p.P;
  const T* qrow = (const T*)p.q + (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride;
  for (int d = lane; d < D; d += 64) qs[w][d] = Elem<T>::load(qrow + d);
  __builtin_amdgcn_wave_barrier();

  float m_run = -INFINITY, l_run = 0.f, oacc[GEN_MAX_D / 64] = {0.f, 0.f};
  const int lid = list_id(p, g, i);
  const int32_t len = list_len(p, lid);
  for (int32_t j = 0; j < len; ++j) {
    const int64_t l = list_at(p, lid, j);
    const int64_t first = l * P;
    if (first > a_i) break;
    const int vis = (int)((a_i - first + 1 < P) ? (a_i - first + 1) : P);
    const T* kb = (const T*)p.k_pool + (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride;
    const T* vb = (const T*)p.v_pool + (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride;
    float pmax = -INFINITY;
    for (int t = lane; t < P; t += 64) {
      float s = -INFINITY;
      if (t < vis) {
        const T* kr = kb + (int64_t)t * p.pool_tok_stride;
        float dot = 0.f;
        for (int d = 0; d < D; ++d) dot += qs[w][d] * Elem<T>::load(kr + d);
        s = p.sm_scale * dot;
      }
      pb[w][t] = s;
      pmax = fmaxf(pmax, s);
    }
    pmax = wave_max(pmax);
    const float m_new = fmaxf(m_run, pmax);
    const float alpha = __expf(m_run - m_new);  // exp(-inf) = 0 on the first page
    float psum = 0.f;
    for (int t = lane; t < P; t += 64) {
      const float pr = (t < vis) ? __expf(pb[w][t] - m_new) : 0.f;
      pb[w][t] = pr;
      psum += pr;
    }
    psum = wave_sum(psum);
    l_run = l_run * alpha + psum;
    m_run = m_new;
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int k = 0; k < GEN_MAX_D / 64; ++k) oacc[k] *= alpha;
    for (int t = 0; t < vis; ++t) {
      const float pr = pb[w][t];
      const T* vr = vb + (int64_t)t * p.pool_tok_stride;
#pragma unroll
      for (int k = 0; k < GEN_MAX_D / 64; ++k) {
        const int d = lane + 64 * k;
        if (d < D) oacc[k] += pr * Elem<T>::load(vr + d);
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
  T* orow = (T*)p.o + (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride;
  const float inv = 1.f / l_run;
#pragma unroll
  for (int k = 0; k < GEN_MAX_D / 64; ++k) {
    const int d = lane + 64 * k;
    if (d < D) Elem<T>::store(orow + d, oacc[k] * inv);
  }
  if (lane == 0) p.lse[(int64_t)h * p.C + i] = m_run + __logf(l_run);
}

template <typename T>
__global__ __launch_bounds__(64 * GEN_WAVES) void dq_generic_kernel(Params p) {
  __shared__ float qs[GEN_WAVES][GEN_MAX_D];
  __shared__ float dos[GEN_WAVES][GEN_MAX_D];
  __shared__ float pb[GEN_WAVES][GEN_MAX_P];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * GEN_WAVES + w;
  if (row >= (int64_t)p.C * p.Hq) return;
  const int i = (int)(row / p.Hq), h = (int)(row % p.Hq), g = h / p.G;
  const int64_t a_i = p.N - p.C + i;
  const int D = p.D, P = p.P;
  const int64_t roff = (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride;
  for (int d = lane; d < D; d += 64) {
    qs[w][d] = Elem<T>::load((const T*)p.q + roff + d);
    dos[w][d] = Elem<T>::load((const T*)p.d_o + roff + d);
  }
  __builtin_amdgcn_wave_barrier();
  const float lse = p.lse[(int64_t)h * p.C + i], delta = p.delta[(int64_t)h * p.C + i];
  float acc[GEN_MAX_D / 64] = {0.f, 0.f};
  const int lid = list_id(p, g, i);
  const int32_t len = list_len(p, lid);
  for (int32_t j = 0; j < len; ++j) {
    const int64_t l = list_at(p, lid, j);
    const int64_t first = l * P;
    if (first > a_i) break;
    const int vis = (int)((a_i - first + 1 < P) ? (a_i - first + 1) : P);
    const T* kb = (const T*)p.k_pool + (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride;
    const T* vb = (const T*)p.v_pool + (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride;
    for (int t = lane; t < vis; t += 64) {
      const T* kr = kb + (int64_t)t * p.pool_tok_stride;
      const T* vr = vb + (int64_t)t * p.pool_tok_stride;
      float dot = 0.f, dp = 0.f;
      for (int d = 0; d < D; ++d) {
        dot += qs[w][d] * Elem<T>::load(kr + d);
        dp += dos[w][d] * Elem<T>::load(vr + d);
      }
      const float pr = __expf(p.sm_scale * dot - lse);
      pb[w][t] = pr * (dp - delta);
    }
    __builtin_amdgcn_wave_barrier();
    for (int t = 0; t < vis; ++t) {
      const float ds = pb[w][t];
      const T* kr = kb + (int64_t)t * p.pool_tok_stride;
#pragma unroll
      for (int k = 0; k < GEN_MAX_D / 64; ++k) {
        const int d = lane + 64 * k;
        if (d < D) acc[k] += ds * Elem<T>::load(kr + d);
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
#pragma unroll
  for (int k = 0; k < GEN_MAX_D / 64; ++k) {
    const int d = lane + 64 * k;
    if (d < D) Elem<T>::store((T*)p.d_q + roff + d, acc[k] * p.sm_scale);
  }
}

// One wave owns one key token of one selected (KV head, page): it visits every
// (head of the group, query row) that sees the token and read-modify-writes the
// token's dK / dV row once.
template <typename T, typename TG>
__global__ __launch_bounds__(64 * GEN_WAVES) void dkv_generic_kernel(Params p) {
  __shared__ float ks[GEN_WAVES][GEN_MAX_D];
  __shared__ float vs[GEN_WAVES][GEN_MAX_D];
  __shared__ float pb[GEN_WAVES][64];
  __shared__ float dsb[GEN_WAVES][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int g = blockIdx.z;
  const int32_t j = blockIdx.y;
  const int t = blockIdx.x * GEN_WAVES + w;
  if (j >= owned_len(p, g) || t >= p.P) return;
  const int D = p.D;
  const int64_t l = owned_at(p, g, j);
  const int64_t pos = l * p.P + t;
  const int64_t koff = (int64_t)p.page_table[l] * p.pool_page_stride + (int64_t)g * p.pool_head_stride +
                       (int64_t)t * p.pool_tok_stride;
  for (int d = lane; d < D; d += 64) {
    ks[w][d] = Elem<T>::load((const T*)p.k_pool + koff + d);
    vs[w][d] = Elem<T>::load((const T*)p.v_pool + koff + d);
  }
  __builtin_amdgcn_wave_barrier();
  const int64_t first_q = p.N - p.C;
  const int i_min = (int)(pos > first_q ? pos - first_q : 0);
  // rows that may see the token.  One list per KV head: every (token >= i_min, head of the group).
  // One list per query page: the rows of the query pages in the page's inverse list.
  const int32_t* inv = nullptr;
  int32_t inv_cnt = 0;
  if (p.qp) {
    const int32_t* off = p.inv_off + (int64_t)g * (p.un_stride + 1) + j;
    inv = p.inv_qp + (int64_t)g * p.m * p.sel_stride + off[0];
    inv_cnt = off[1] - off[0];
  }
  const int64_t n_rows = p.qp ? (int64_t)inv_cnt * p.P * p.G : (int64_t)(p.C - i_min) * p.G;
  auto row_of = [&](int64_t rr, int& i, int& h) -> bool {
    if (!p.qp) {
      i = i_min + (int)(rr / p.G);
      h = g * p.G + (int)(rr % p.G);
      return true;
    }
    const int32_t pg = p.P * p.G, q = (int32_t)(rr / pg), rem = (int32_t)(rr % pg);
    i = inv[q] * p.P + rem / p.G;
    h = g * p.G + rem % p.G;
    return i >= i_min;
  };
  float dk[GEN_MAX_D / 64] = {0.f, 0.f}, dv[GEN_MAX_D / 64] = {0.f, 0.f};
  for (int64_t r0 = 0; r0 < n_rows; r0 += 64) {
    const int64_t rr = r0 + lane;
    float pr = 0.f, ds = 0.f;
    int i = 0, h = 0;
    if (rr < n_rows && row_of(rr, i, h)) {
      const int64_t roff = (int64_t)i * p.q_tok_stride + (int64_t)h * p.q_head_stride;
      float dot = 0.f, dp = 0.f;
      for (int d = 0; d < D; ++d) {
        dot += ks[w][d] * Elem<T>::load((const T*)p.q + roff + d);
        dp += vs[w][d] * Elem<T>::load((const T*)p.d_o + roff + d);
      }
      pr = __expf(p.sm_scale * dot - p.lse[(int64_t)h * p.C + i]);
      ds = pr * (dp - p.delta[(int64_t)h * p.C + i]);
    }
    pb[w][lane] = pr;
    dsb[w][lane] = ds;
    __builtin_amdgcn_wave_barrier();
    const int cnt = (int)((n_rows - r0 < 64) ? (n_rows - r0) : 64);
    for (int x = 0; x < cnt; ++x) {
      int i2 = 0, h2 = 0;
      if (!row_of(r0 + x, i2, h2)) continue;  // (wave-uniform)
      const int64_t roff = (int64_t)i2 * p.q_tok_stride + (int64_t)h2 * p.q_head_stride;
      const float a = pb[w][x], b = dsb[w][x];
#pragma unroll
      for (int k = 0; k < GEN_MAX_D / 64; ++k) {
        const int d = lane + 64 * k;
        if (d < D) {
          dv[k] += a * Elem<T>::load((const T*)p.d_o + roff + d);
          dk[k] += b * Elem<T>::load((const T*)p.q + roff + d);
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
#pragma unroll
  for (int k = 0; k < GEN_MAX_D / 64; ++k) {
    const int d = lane + 64 * k;
    if (d < D) {
      TG* pk = (TG*)p.dk_pool + koff + d;
      TG* pv = (TG*)p.dv_pool + koff + d;
      Elem<TG>::store(pk, Elem<TG>::load(pk) + p.sm_scale * dk[k]);
      Elem<TG>::store(pv, Elem<TG>::load(pv) + dv[k]);
    }
  }
}

hipError_t launch_delta(const Params& p, bool is_bf16, hipStream_t st) {
  const int64_t rows = (int64_t)p.C * p.Hq;
  dim3 grid((unsigned)((rows + 3) / 4));
  ProfScope prof_("delta", st);
  if (is_bf16) delta_kernel<bf16_t><<<grid, dim3(256), 0, st>>>(p);
  else delta_kernel<float><<<grid, dim3(256), 0, st>>>(p);
  return hipGetLastError();
}

hipError_t launch_fwd_generic(const Params& p, bool is_bf16, hipStream_t st) {
  const int64_t rows = (int64_t)p.C * p.Hq;
  dim3 grid((unsigned)((rows + GEN_WAVES - 1) / GEN_WAVES));
  ProfScope prof_("attn_fwd_generic", st);
  if (is_bf16) fwd_generic_kernel<bf16_t><<<grid, dim3(64 * GEN_WAVES), 0, st>>>(p);
  else fwd_generic_kernel<float><<<grid, dim3(64 * GEN_WAVES), 0, st>>>(p);
  return hipGetLastError();
}

// max_list_len: host-side upper bound of the per-head list length (grid size).
hipError_t launch_bwd_generic(const Params& p, bool is_bf16, int32_t max_list_len, hipStream_t st) {
  const int64_t rows = (int64_t)p.C * p.Hq;
  dim3 grid((unsigned)((rows + GEN_WAVES - 1) / GEN_WAVES));
  dim3 gkv((unsigned)((p.P + GEN_WAVES - 1) / GEN_WAVES), (unsigned)max_list_len, (unsigned)p.Hkv);
  dim3 blk(64 * GEN_WAVES);
  ProfScope prof_("attn_bwd_generic", st);
  if (is_bf16) {
    dq_generic_kernel<bf16_t><<<grid, blk, 0, st>>>(p);
    if (p.grad_is_bf16) dkv_generic_kernel<bf16_t, bf16_t><<<gkv, blk, 0, st>>>(p);
    else dkv_generic_kernel<bf16_t, float><<<gkv, blk, 0, st>>>(p);
  } else {
    dq_generic_kernel<float><<<grid, blk, 0, st>>>(p);
    if (p.grad_is_bf16) dkv_generic_kernel<float, bf16_t><<<gkv, blk, 0, st>>>(p);
    else dkv_generic_kernel<float, float><<<gkv, blk, 0, st>>>(p);
  }
  return hipGetLastError();
}

}  // namespace oomb
