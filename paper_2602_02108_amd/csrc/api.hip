// C-ABI entry points: host-side validation and kernel dispatch.  Nothing is
// allocated, freed or synchronised here; every launch goes to the caller's stream.
#include <cmath>
#include <cstdlib>

#include "common.h"
#include "launch.h"

using namespace oomb;

namespace {

bool is_pow2(int64_t x) { return x > 0 && (x & (x - 1)) == 0; }
size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }
size_t elem_size(int32_t dt) { return dt == OOMB_BF16 ? 2 : 4; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Kernels without MFMA can be forced for debugging and cross-checks.
bool force_generic() {
  static int v = -1;
  if (v < 0) {
    const char* e = std::getenv("OOMB_FORCE_GENERIC");
    v = (e && e[0] == '1') ? 1 : 0;
  }
  return v == 1;
}

oomb_status check_desc(const oomb_attn_desc* d, Params* p) {
  if (!d) return OOMB_ERR_INVALID_ARG;
  if (d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->n_q_heads % d->n_kv_heads) return OOMB_ERR_INVALID_ARG;
  if (d->head_dim <= 0 || d->page_size <= 0 || d->chunk_len <= 0 || d->ctx_len <= 0) return OOMB_ERR_INVALID_ARG;
  if (d->chunk_len % d->page_size || d->ctx_len % d->page_size || d->ctx_len < d->chunk_len)
    return OOMB_ERR_INVALID_ARG;
  if ((d->dtype != OOMB_F32 && d->dtype != OOMB_BF16) || (d->grad_dtype != OOMB_F32 && d->grad_dtype != OOMB_BF16))
    return OOMB_ERR_INVALID_ARG;
  if (!(d->sm_scale > 0.f) || !std::isfinite(d->sm_scale)) return OOMB_ERR_INVALID_ARG;
  const size_t es = elem_size(d->dtype), gs = elem_size(d->grad_dtype);
  const int64_t strides[5] = {d->pool_page_stride, d->pool_head_stride, d->pool_tok_stride, d->q_tok_stride,
                              d->q_head_stride};
  for (int64_t s : strides) {
    if (s < d->head_dim) return OOMB_ERR_INVALID_ARG;
    if ((s * (int64_t)es) % 16 || (s * (int64_t)gs) % 16) return OOMB_ERR_INVALID_ARG;
  }
  if (d->num_phys_pages < d->ctx_len / d->page_size) return OOMB_ERR_INVALID_ARG;
  if (d->ctx_len / d->page_size > INT32_MAX) return OOMB_ERR_INVALID_ARG;
  if ((d->head_dim != 64 && d->head_dim != 128) || !is_pow2(d->page_size) || d->page_size < 16 ||
      d->page_size > 128)
    return OOMB_ERR_UNSUPPORTED;
  p->Hq = d->n_q_heads; p->Hkv = d->n_kv_heads; p->G = p->Hq / p->Hkv; p->D = d->head_dim;
  p->P = d->page_size; p->C = d->chunk_len; p->m = p->C / p->P;
  p->N = d->ctx_len; p->n = p->N / p->P; p->n_past = p->n - p->m;
  p->sm_scale = d->sm_scale;
  p->pool_page_stride = d->pool_page_stride; p->pool_head_stride = d->pool_head_stride;
  p->pool_tok_stride = d->pool_tok_stride;
  p->q_tok_stride = d->q_tok_stride; p->q_head_stride = d->q_head_stride;
  p->grad_is_bf16 = d->grad_dtype == OOMB_BF16;
  p->g_magic = p->G > 1 ? (uint32_t)(((1ull << 32) + (uint64_t)p->G - 1) / (uint64_t)p->G) : 0u;
  if ((int64_t)p->C * p->G >= (1ll << 31) / p->G) return OOMB_ERR_UNSUPPORTED;
  return OOMB_OK;
}

oomb_status check_list(const Params& p, const int32_t* sel, const int32_t* cnt, int32_t stride,
                       int32_t* max_len) {
  if (!sel) {
    *max_len = (int32_t)p.n;
    return OOMB_OK;
  }
  if (!cnt || stride < p.m) return OOMB_ERR_INVALID_ARG;
  *max_len = stride < p.n ? stride : (int32_t)p.n;
  return OOMB_OK;
}

// One list per (KV head, query page): [maps derived from the lists][what the kernels need with the
// union of a KV head's lists in the place of its list].  p.sel_stride is set here.
size_t qp_workspace_bytes(Params p, int32_t stride, bool bf, bool bwd) {
  p.qp = 1;
  p.sel_stride = stride;
  const size_t maps = qp_maps_bytes(p, stride);
  const int32_t cap = qp_union_cap(p, stride);
  if (!force_generic() && mfma_supported(p, bf))
    return maps + (bwd ? bwd_mfma_workspace_bytes(p, cap) : fwd_mfma_workspace_bytes(p, cap));
  return maps + (bwd ? up256((size_t)p.Hq * p.C * sizeof(float)) : 256);
}

oomb_status check_qp_list(const Params& p, const int32_t* sel, const int32_t* cnt, int32_t stride) {
  if (!sel || !cnt || stride < p.m) return OOMB_ERR_INVALID_ARG;
  if ((int64_t)stride * p.m > INT32_MAX) return OOMB_ERR_UNSUPPORTED;
  return OOMB_OK;
}

}  // namespace

extern "C" {

size_t oomb_workspace_bytes(const oomb_attn_desc* desc, int32_t top_k, int32_t op) {
  Params p{};
  if (check_desc(desc, &p) != OOMB_OK) return 0;
  switch (op) {
    case OOMB_OP_SCORE_TOPK:
      if (top_k < 0) return 0;
      return score_workspace_bytes(p);
    case OOMB_OP_ATTN_FWD: {
      int64_t max_len = p.n;
      if (top_k >= 0 && (int64_t)top_k + p.m < max_len) max_len = (int64_t)top_k + p.m;
      const size_t mfma = mfma_supported(p, desc->dtype == OOMB_BF16) ? fwd_mfma_workspace_bytes(p, (int32_t)max_len) : 0;
      return mfma > 256 ? mfma : 256;
    }
    case OOMB_OP_ATTN_BWD: {
      // longest selection list the call may be given: top_k retrieved pages + the m local pages
      int64_t max_len = p.n;
      if (top_k >= 0 && (int64_t)top_k + p.m < max_len) max_len = (int64_t)top_k + p.m;
      const size_t generic = up256((size_t)p.Hq * p.C * sizeof(float));
      const size_t mfma = mfma_supported(p, desc->dtype == OOMB_BF16) ? bwd_mfma_workspace_bytes(p, (int32_t)max_len) : 0;
      return generic > mfma ? generic : mfma;
    }
    case OOMB_OP_VOTE_TOPK:
      if (top_k < 0) return 0;
      return vote_workspace_bytes(p, desc->dtype == OOMB_BF16, force_generic());
    case OOMB_OP_CHECK_INPUTS:
      return up256((size_t)desc->num_phys_pages * sizeof(int32_t));
    case OOMB_OP_ATTN_FWD_QP:
    case OOMB_OP_ATTN_BWD_QP: {
      if (top_k < 0) return 0;
      const int64_t stride = (int64_t)top_k + p.m;
      if (stride * p.m > INT32_MAX) return 0;
      return qp_workspace_bytes(p, (int32_t)stride, desc->dtype == OOMB_BF16, op == OOMB_OP_ATTN_BWD_QP);
    }
    default:
      return 0;
  }
}

oomb_status oomb_page_score_topk(const oomb_attn_desc* desc, const void* q, const void* k_pool,
                                 const int32_t* page_table, int32_t top_k, int32_t* sel_pages,
                                 int32_t* sel_count, float* scores_out, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!q || !k_pool || !page_table || !sel_pages || !sel_count || top_k < 0) return OOMB_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_pool)) return OOMB_ERR_INVALID_ARG;
  if (p.n_past > (1 << 20)) return OOMB_ERR_UNSUPPORTED;
  if (!workspace || workspace_bytes < score_workspace_bytes(p)) return OOMB_ERR_WORKSPACE;
  p.q = q; p.k_pool = k_pool; p.page_table = page_table;
  hipError_t e = launch_score_topk(p, desc->dtype == OOMB_BF16, top_k, sel_pages, sel_count, scores_out,
                                   workspace, nullptr, (hipStream_t)hip_stream);
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

oomb_status oomb_page_score_topk_noalloc(const oomb_attn_desc* desc, const void* q, const void* k_pool,
                                         const int32_t* page_table, int32_t top_k, int32_t* sel_pages,
                                         int32_t* sel_count, float* scores_out, void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!q || !k_pool || !page_table || !sel_pages || !sel_count || top_k < 0) return OOMB_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_pool)) return OOMB_ERR_INVALID_ARG;
  if (p.n_past > (1 << 20)) return OOMB_ERR_UNSUPPORTED;
  if (score_workspace_bytes(p) > (size_t)OOMB_NOALLOC_SCRATCH_BYTES) return OOMB_ERR_SCRATCH_LIMIT;
  void* ws = nullptr;
  if (score_scratch_ptr(&ws) != hipSuccess) return OOMB_ERR_LAUNCH;
  p.q = q; p.k_pool = k_pool; p.page_table = page_table;
  hipError_t e = launch_score_topk(p, desc->dtype == OOMB_BF16, top_k, sel_pages, sel_count, scores_out, ws, nullptr,
                                   (hipStream_t)hip_stream);
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

oomb_status oomb_page_score_topk_cached(const oomb_attn_desc* desc, const void* q, const float* kbar_cache,
                                        int32_t top_k, int32_t* sel_pages, int32_t* sel_count, float* scores_out,
                                        void* workspace, size_t workspace_bytes, void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!q || !kbar_cache || !sel_pages || !sel_count || top_k < 0) return OOMB_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(kbar_cache)) return OOMB_ERR_INVALID_ARG;
  if (p.n_past > (1 << 20)) return OOMB_ERR_UNSUPPORTED;
  if (!workspace || workspace_bytes < score_workspace_bytes(p)) return OOMB_ERR_WORKSPACE;
  p.q = q;
  hipError_t e = launch_score_topk(p, desc->dtype == OOMB_BF16, top_k, sel_pages, sel_count, scores_out,
                                   workspace, kbar_cache, (hipStream_t)hip_stream);
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

oomb_status oomb_kv_append(const oomb_attn_desc* desc, const void* k_chunk, const void* v_chunk,
                           const int32_t* page_table, void* k_pool, void* v_pool, float* kbar_cache,
                           void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!k_chunk || !v_chunk || !page_table || !k_pool || !v_pool) return OOMB_ERR_INVALID_ARG;
  if (!aligned16(k_chunk) || !aligned16(v_chunk) || !aligned16(k_pool) || !aligned16(v_pool) ||
      (kbar_cache && !aligned16(kbar_cache)))
    return OOMB_ERR_INVALID_ARG;
  p.page_table = page_table;
  p.k_pool = k_pool;
  hipError_t e = launch_kv_append(p, desc->dtype == OOMB_BF16, k_chunk, v_chunk, k_pool, v_pool, kbar_cache,
                                  (hipStream_t)hip_stream);
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

oomb_status oomb_page_means(const oomb_attn_desc* desc, const void* k_pool, const int32_t* page_table,
                            int64_t first_page, int64_t n_pages, float* kbar_cache, void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!k_pool || !page_table || !kbar_cache || first_page < 0 || n_pages < 0 || first_page + n_pages > p.n)
    return OOMB_ERR_INVALID_ARG;
  if (!aligned16(k_pool) || !aligned16(kbar_cache)) return OOMB_ERR_INVALID_ARG;
  p.page_table = page_table;
  p.k_pool = k_pool;
  hipError_t e = launch_page_means(p, desc->dtype == OOMB_BF16, first_page, n_pages, kbar_cache, (hipStream_t)hip_stream);
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

oomb_status oomb_local_page_list(const oomb_attn_desc* desc, int32_t window_pages, int32_t* sel_pages,
                                 int32_t* sel_count, void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!sel_pages || !sel_count || window_pages < 0) return OOMB_ERR_INVALID_ARG;
  hipError_t e = launch_local_page_list(p, window_pages, sel_pages, sel_count, (hipStream_t)hip_stream);
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

oomb_status oomb_paged_attn_fwd(const oomb_attn_desc* desc, const void* q, const void* k_pool,
                                const void* v_pool, const int32_t* page_table,
                                const int32_t* sel_pages, const int32_t* sel_count,
                                int32_t sel_stride, void* o, float* lse, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!q || !k_pool || !v_pool || !page_table || !o || !lse) return OOMB_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(o)) return OOMB_ERR_INVALID_ARG;
  int32_t max_len = 0;
  s = check_list(p, sel_pages, sel_count, sel_stride, &max_len);
  if (s != OOMB_OK) return s;
  p.q = q; p.k_pool = k_pool; p.v_pool = v_pool; p.page_table = page_table;
  p.sel = sel_pages; p.sel_count = sel_count; p.sel_stride = sel_stride;
  p.o = o; p.lse = lse;
  const bool bf = desc->dtype == OOMB_BF16;
  hipError_t e;
  if (!force_generic() && mfma_supported(p, bf)) {
    if (!workspace || workspace_bytes < fwd_mfma_workspace_bytes(p, max_len) || !aligned16(workspace))
      return OOMB_ERR_WORKSPACE;
    e = launch_fwd_mfma(p, max_len, workspace, (hipStream_t)hip_stream);
  } else {
    e = launch_fwd_generic(p, bf, (hipStream_t)hip_stream);
  }
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

oomb_status oomb_paged_attn_bwd(const oomb_attn_desc* desc, const void* q, const void* k_pool,
                                const void* v_pool, const int32_t* page_table,
                                const int32_t* sel_pages, const int32_t* sel_count,
                                int32_t sel_stride, const void* o, const float* lse,
                                const void* d_o, void* d_q, void* dk_pool, void* dv_pool,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!q || !k_pool || !v_pool || !page_table || !o || !lse || !d_o || !d_q || !dk_pool || !dv_pool)
    return OOMB_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(o) || !aligned16(d_o) ||
      !aligned16(d_q) || !aligned16(dk_pool) || !aligned16(dv_pool))
    return OOMB_ERR_INVALID_ARG;
  int32_t max_len = 0;
  s = check_list(p, sel_pages, sel_count, sel_stride, &max_len);
  if (s != OOMB_OK) return s;
  const bool bf = desc->dtype == OOMB_BF16;
  const bool use_mfma = !force_generic() && mfma_supported(p, bf);
  // the shape-generic dK/dV kernel walks the list entries in a grid dimension of at most 65535
  if (!use_mfma && (max_len > 65535 || p.Hkv > 65535)) return OOMB_ERR_UNSUPPORTED;
  const size_t need = use_mfma ? bwd_mfma_workspace_bytes(p, max_len) : up256((size_t)p.Hq * p.C * sizeof(float));
  if (!workspace || workspace_bytes < need || !aligned16(workspace)) return OOMB_ERR_WORKSPACE;
  p.q = q; p.k_pool = k_pool; p.v_pool = v_pool; p.page_table = page_table;
  p.sel = sel_pages; p.sel_count = sel_count; p.sel_stride = sel_stride;
  p.o = const_cast<void*>(o); p.lse = const_cast<float*>(lse); p.d_o = d_o; p.d_q = d_q;
  p.dk_pool = dk_pool; p.dv_pool = dv_pool;
  p.delta = (float*)workspace;
  hipStream_t st = (hipStream_t)hip_stream;
  hipError_t e;
  if (use_mfma) {
    e = launch_bwd_mfma(p, max_len, workspace, st);
  } else {
    e = launch_delta(p, bf, st);
    if (e != hipSuccess) return OOMB_ERR_LAUNCH;
    e = launch_bwd_generic(p, bf, max_len, st);
  }
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

oomb_status oomb_page_vote_topk(const oomb_attn_desc* desc, const void* q, const float* kbar_cache, int32_t top_k,
                                int32_t* sel_pages, int32_t* sel_count, float* votes_out, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!q || !kbar_cache || !sel_pages || !sel_count || top_k < 0) return OOMB_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(kbar_cache)) return OOMB_ERR_INVALID_ARG;
  if (p.n_past > (1 << 20) || (int64_t)p.Hkv * p.m > 65535) return OOMB_ERR_UNSUPPORTED;
  const bool bf = desc->dtype == OOMB_BF16;
  if (!workspace || workspace_bytes < vote_workspace_bytes(p, bf, force_generic()) || !aligned16(workspace))
    return OOMB_ERR_WORKSPACE;
  p.q = q;
  hipError_t e = launch_vote_topk(p, bf, force_generic(), kbar_cache, top_k, sel_pages, sel_count, votes_out, workspace,
                                  (hipStream_t)hip_stream);
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

oomb_status oomb_paged_attn_fwd_qp(const oomb_attn_desc* desc, const void* q, const void* k_pool,
                                   const void* v_pool, const int32_t* page_table,
                                   const int32_t* sel_pages, const int32_t* sel_count,
                                   int32_t sel_stride, void* o, float* lse, void* workspace,
                                   size_t workspace_bytes, void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!q || !k_pool || !v_pool || !page_table || !o || !lse) return OOMB_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(o)) return OOMB_ERR_INVALID_ARG;
  s = check_qp_list(p, sel_pages, sel_count, sel_stride);
  if (s != OOMB_OK) return s;
  const bool bf = desc->dtype == OOMB_BF16;
  if (!workspace || workspace_bytes < qp_workspace_bytes(p, sel_stride, bf, false) || !aligned16(workspace))
    return OOMB_ERR_WORKSPACE;
  p.q = q; p.k_pool = k_pool; p.v_pool = v_pool; p.page_table = page_table;
  p.sel = sel_pages; p.sel_count = sel_count; p.sel_stride = sel_stride;
  p.o = o; p.lse = lse;
  p.qp = 1;
  hipStream_t st = (hipStream_t)hip_stream;
  hipError_t e;
  if (!force_generic() && mfma_supported(p, bf)) {
    e = launch_qp_prepare(p, workspace, st);
    if (e != hipSuccess) return OOMB_ERR_LAUNCH;
    e = launch_fwd_mfma(p, qp_union_cap(p, sel_stride), (unsigned char*)workspace + qp_maps_bytes(p, sel_stride), st);
  } else {
    e = launch_fwd_generic(p, bf, st);
  }
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

oomb_status oomb_paged_attn_bwd_qp(const oomb_attn_desc* desc, const void* q, const void* k_pool,
                                   const void* v_pool, const int32_t* page_table,
                                   const int32_t* sel_pages, const int32_t* sel_count,
                                   int32_t sel_stride, const void* o, const float* lse,
                                   const void* d_o, void* d_q, void* dk_pool, void* dv_pool,
                                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!q || !k_pool || !v_pool || !page_table || !o || !lse || !d_o || !d_q || !dk_pool || !dv_pool)
    return OOMB_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(o) || !aligned16(d_o) ||
      !aligned16(d_q) || !aligned16(dk_pool) || !aligned16(dv_pool))
    return OOMB_ERR_INVALID_ARG;
  s = check_qp_list(p, sel_pages, sel_count, sel_stride);
  if (s != OOMB_OK) return s;
  const bool bf = desc->dtype == OOMB_BF16;
  const bool use_mfma = !force_generic() && mfma_supported(p, bf);
  // grid dimensions of at most 65535: list entries of the shape-generic dK/dV kernel, cut pages of the slice reduction
  if (p.Hkv > 65535 || (!use_mfma && qp_union_cap(p, sel_stride) > 65535) ||
      (use_mfma && qp_max_multi(p, sel_stride) > 65535))
    return OOMB_ERR_UNSUPPORTED;
  if (!workspace || workspace_bytes < qp_workspace_bytes(p, sel_stride, bf, true) || !aligned16(workspace))
    return OOMB_ERR_WORKSPACE;
  p.q = q; p.k_pool = k_pool; p.v_pool = v_pool; p.page_table = page_table;
  p.sel = sel_pages; p.sel_count = sel_count; p.sel_stride = sel_stride;
  p.o = const_cast<void*>(o); p.lse = const_cast<float*>(lse); p.d_o = d_o; p.d_q = d_q;
  p.dk_pool = dk_pool; p.dv_pool = dv_pool;
  hipStream_t st = (hipStream_t)hip_stream;
  hipError_t e = launch_qp_prepare(p, workspace, st);
  if (e != hipSuccess) return OOMB_ERR_LAUNCH;
  unsigned char* rest = (unsigned char*)workspace + qp_maps_bytes(p, sel_stride);
  const int32_t cap = qp_union_cap(p, sel_stride);
  if (use_mfma) {
    e = launch_bwd_mfma(p, cap, rest, st);
  } else {
    p.delta = (float*)rest;
    e = launch_delta(p, bf, st);
    if (e != hipSuccess) return OOMB_ERR_LAUNCH;
    e = launch_bwd_generic(p, bf, cap, st);
  }
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

oomb_status oomb_offload_plan(const oomb_attn_desc* desc, const int32_t* sel_pages, const int32_t* sel_count,
                              int32_t sel_stride, int32_t lists_per_head, int32_t stage_capacity, int32_t* stage_table,
                              int32_t* slot_pages, uint32_t* head_mask, int32_t* n_slots, void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!sel_pages || !sel_count || sel_stride < p.m || stage_capacity <= 0 || !stage_table || !slot_pages || !head_mask ||
      !n_slots)
    return OOMB_ERR_INVALID_ARG;
  if (lists_per_head != 1 && lists_per_head != p.m) return OOMB_ERR_INVALID_ARG;
  if (p.Hkv > 32 || (int64_t)lists_per_head * sel_stride > INT32_MAX) return OOMB_ERR_UNSUPPORTED;
  p.sel = sel_pages; p.sel_count = sel_count; p.sel_stride = sel_stride;
  hipError_t e = launch_offload_plan(p, lists_per_head, stage_capacity, stage_table, slot_pages, head_mask, n_slots,
                                     (hipStream_t)hip_stream);
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

oomb_status oomb_offload_fetch(const oomb_attn_desc* desc, const void* host_k_pool, const void* host_v_pool,
                               const int32_t* page_table, const int32_t* slot_pages, const uint32_t* head_mask,
                               const int32_t* n_slots, int32_t stage_capacity, void* stage_k, void* stage_v,
                               void* stage_dk, void* stage_dv, void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!host_k_pool || !host_v_pool || !page_table || !slot_pages || !head_mask || !n_slots || stage_capacity <= 0 ||
      !stage_k || !stage_v || (stage_dk == nullptr) != (stage_dv == nullptr))
    return OOMB_ERR_INVALID_ARG;
  if (!aligned16(host_k_pool) || !aligned16(host_v_pool) || !aligned16(stage_k) || !aligned16(stage_v) ||
      !aligned16(stage_dk) || !aligned16(stage_dv))
    return OOMB_ERR_INVALID_ARG;
  // the kernels dereference the host pools: they must be memory the device can reach
  void* hk = device_view(host_k_pool);
  void* hv = device_view(host_v_pool);
  if (!hk || !hv) return OOMB_ERR_INVALID_ARG;
  p.page_table = page_table;
  hipError_t e = launch_offload_fetch(p, desc->dtype == OOMB_BF16, slot_pages, head_mask, n_slots, stage_capacity, hk, hv,
                                      stage_k, stage_v, stage_dk, stage_dv, (hipStream_t)hip_stream);
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

oomb_status oomb_offload_writeback(const oomb_attn_desc* desc, const void* stage_dk, const void* stage_dv,
                                   void* host_dk_pool, void* host_dv_pool, const int32_t* page_table,
                                   const int32_t* slot_pages, const uint32_t* head_mask, const int32_t* n_slots,
                                   int32_t stage_capacity, void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!stage_dk || !stage_dv || !host_dk_pool || !host_dv_pool || !page_table || !slot_pages || !head_mask || !n_slots ||
      stage_capacity <= 0)
    return OOMB_ERR_INVALID_ARG;
  if (!aligned16(stage_dk) || !aligned16(stage_dv) || !aligned16(host_dk_pool) || !aligned16(host_dv_pool))
    return OOMB_ERR_INVALID_ARG;
  void* hk = device_view(host_dk_pool);
  void* hv = device_view(host_dv_pool);
  if (!hk || !hv) return OOMB_ERR_INVALID_ARG;
  p.page_table = page_table;
  hipError_t e = launch_offload_writeback(p, slot_pages, head_mask, n_slots, stage_capacity, const_cast<void*>(stage_dk),
                                          const_cast<void*>(stage_dv), hk, hv, (hipStream_t)hip_stream);
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

oomb_status oomb_check_inputs(const oomb_attn_desc* desc, const int32_t* page_table, const int32_t* sel_pages,
                              const int32_t* sel_count, int32_t sel_stride, int32_t lists_per_head, int32_t* violations,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
  Params p{};
  oomb_status s = check_desc(desc, &p);
  if (s != OOMB_OK) return s;
  if (!page_table || !violations) return OOMB_ERR_INVALID_ARG;
  if (sel_pages) {
    if (!sel_count || sel_stride < 1 || (lists_per_head != 1 && lists_per_head != p.m)) return OOMB_ERR_INVALID_ARG;
  } else {
    lists_per_head = 0;
  }
  if (!workspace || workspace_bytes < up256((size_t)desc->num_phys_pages * sizeof(int32_t))) return OOMB_ERR_WORKSPACE;
  p.page_table = page_table;
  p.sel = sel_pages; p.sel_count = sel_count; p.sel_stride = sel_stride;
  hipError_t e = launch_check_inputs(p, desc->num_phys_pages, lists_per_head, (int32_t*)workspace, violations,
                                     (hipStream_t)hip_stream);
  return e == hipSuccess ? OOMB_OK : OOMB_ERR_LAUNCH;
}

const char* oomb_status_string(int32_t status) {
  switch (status) {
    case OOMB_OK: return "ok";
    case OOMB_ERR_INVALID_ARG: return "invalid argument";
    case OOMB_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case OOMB_ERR_WORKSPACE: return "workspace missing or too small";
    case OOMB_ERR_LAUNCH: return "kernel launch failed";
    case OOMB_ERR_OUT_OF_PAGES: return "page pool exhausted";
    case OOMB_ERR_SCRATCH_LIMIT: return "shape exceeds the built-in scratch buffer";
    default: return "unknown status";
  }
}

int32_t oomb_version(void) { return 200; }

}  // extern "C"
