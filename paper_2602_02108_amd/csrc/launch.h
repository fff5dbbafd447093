// Host-side entry points of the kernel files: what api.hip dispatches to, and the few helpers the
// kernel files share among themselves.  Every launch_* only enqueues work on the given stream and
// returns hipGetLastError(); the *_bytes functions size the caller-owned workspaces.
#pragma once
#include "common.h"

namespace oomb {

// score_topk.hip: pooled query, page scores (from the keys or from cached page means), top-k lists
size_t score_workspace_bytes(const Params& p);
hipError_t launch_score_topk(const Params& p, bool is_bf16, int32_t top_k, int32_t* sel, int32_t* sel_count,
                             float* scores_out, void* ws, const float* kbar_cache, hipStream_t st);
hipError_t score_scratch_ptr(void** out);  // this device's copy of the built-in scoring scratch array
hipError_t launch_topk_select_qp(const Params& p, const float* votes, int32_t top_k, int32_t* sel, int32_t* sel_count,
                                 hipStream_t st);

// kv_manager.hip: append, page means, scores from cached means, page list of a local-attention layer
hipError_t launch_kv_append(const Params& p, bool is_bf16, const void* kc, const void* vc, void* k_pool, void* v_pool,
                            float* cache, hipStream_t st);
hipError_t launch_page_means(const Params& p, bool is_bf16, int64_t first, int64_t count, float* cache, hipStream_t st);
hipError_t launch_page_score_cached(const Params& p, const float* qbar, const float* cache, float* scores, hipStream_t st);
hipError_t launch_local_page_list(const Params& p, int32_t window, int32_t* sel, int32_t* sel_count, hipStream_t st);

// vote_topk.hip: votes per query page and their lists
size_t vote_workspace_bytes(const Params& p, bool is_bf16, bool force_generic);
hipError_t launch_vote_topk(Params p, bool is_bf16, bool force_generic, const float* kbar, int32_t top_k, int32_t* sel,
                            int32_t* sel_count, float* votes_out, void* ws, hipStream_t st);

// qp_lists.hip: union / inverse lists and dK/dV work units of per-query-page lists
size_t qp_maps_bytes(const Params& p, int32_t stride);
int32_t qp_union_cap(const Params& p, int32_t stride);
int32_t qp_max_units(const Params& p, int32_t stride);
int32_t qp_max_pslots(const Params& p, int32_t stride);
int32_t qp_max_multi(const Params& p, int32_t stride);
hipError_t launch_qp_prepare(Params& p, void* ws, hipStream_t st);

// attn_generic.hip: fp32 tensors and shapes without a matrix-core kernel
hipError_t launch_delta(const Params& p, bool is_bf16, hipStream_t st);
hipError_t launch_fwd_generic(const Params& p, bool is_bf16, hipStream_t st);
hipError_t launch_bwd_generic(const Params& p, bool is_bf16, int32_t max_list_len, hipStream_t st);

// kv_layout.hip: LDS-ordered images of the selected pages
size_t kv_image_bytes(const Params& p, int32_t max_len);
hipError_t launch_kv_layout(const Params& p, int32_t max_len, void* img, hipStream_t st);

// attn_fwd_mfma.hip, attn_bwd_mfma.hip, attn_bwd_dkv_mfma.hip: the matrix-core kernels
bool mfma_supported(const Params& p, bool is_bf16);
size_t fwd_mfma_workspace_bytes(const Params& p, int32_t max_list_len);
hipError_t launch_fwd_mfma(const Params& p, int32_t max_list_len, void* ws, hipStream_t st);
size_t bwd_mfma_workspace_bytes(const Params& p, int32_t max_list_len);
hipError_t launch_bwd_mfma(const Params& p, int32_t max_list_len, void* ws, hipStream_t st);
size_t dkv_partial_bytes(const Params& p, int32_t max_len, int32_t n_split);
int32_t dkv_splits(const Params& p, int32_t max_len);
hipError_t launch_bwd_dkv_mfma(const Params& p, const float* bias, int32_t n_stages, int32_t max_len,
                               float* partial_ws, hipStream_t st);

// offload.hip: staging plan and transfers between pinned host pools and device staging pools
void* device_view(const void* ptr);
hipError_t launch_offload_plan(const Params& p, int32_t lists_per_head, int32_t stage_cap, int32_t* stage_table,
                               int32_t* slot_pages, uint32_t* head_mask, int32_t* n_slots, hipStream_t st);
hipError_t launch_offload_fetch(const Params& p, bool is_bf16, const int32_t* slot_pages, const uint32_t* head_mask,
                                const int32_t* n_slots, int32_t stage_cap, void* host_k, void* host_v, void* stage_k,
                                void* stage_v, void* stage_dk, void* stage_dv, hipStream_t st);
hipError_t launch_offload_writeback(const Params& p, const int32_t* slot_pages, const uint32_t* head_mask,
                                    const int32_t* n_slots, int32_t stage_cap, void* stage_dk, void* stage_dv, void* host_dk,
                                    void* host_dv, hipStream_t st);

// check.hip: debug check of the documented preconditions
hipError_t launch_check_inputs(const Params& p, int64_t num_phys, int32_t lists_per_head, int32_t* marks, int32_t* out,
                               hipStream_t st);

}  // namespace oomb
