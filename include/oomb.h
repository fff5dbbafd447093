/*
 * oomb.h — C ABI of the MI355X (gfx950) paged sparse attention library.
 *
 * The library implements the per-layer hot path of OOMB's chunk-recurrent
 * long-context training: attention of one query chunk against a growing paged
 * KV cache with page-level top-k page selection, forward and backward, the
 * backward accumulating dK/dV in place into a paged KV-gradient pool.
 *
 * Problem statement (paper Sec. 3, Eq. 2-3; Sec. 4.1; Sec. 4.2), notation:
 *   Hq query heads, Hkv KV heads, G = Hq / Hkv, head dim D, page size P,
 *   chunk of C = m*P query tokens, N = n*P tokens reachable through the page
 *   table at call time INCLUDING the chunk's own C tokens as the last m logical
 *   pages, n_past = n - m.  Query head h reads KV head g = h / G.  Query i of
 *   the chunk sits at absolute position a_i = N - C + i and sees token t iff
 *   t <= a_i and logical page t / P is in the selection list of KV head g.
 *
 * Memory: EVERY pointer below is DEVICE memory owned by the caller (except the
 * descriptor, which is host memory read during the call).  No entry point of this
 * header allocates, frees or synchronises; all work is enqueued on `hip_stream`
 * (a hipStream_t; NULL = the default stream) and the call returns at once.  (The
 * benchmark aids of oomb_bench.h -- per-kernel event timing, measured ceilings --
 * are kept apart because they do wait for the device.)
 * Layouts (element strides given in the descriptor, D always contiguous):
 *   Q, O, dO, dQ      [C][Hq][D]       q_tok_stride, q_head_stride
 *   K/V pools         [n_phys][Hkv][P][D]  pool_page_stride, pool_head_stride, pool_tok_stride
 *   dK/dV pools       same strides as the K/V pools, element type grad_dtype
 *   page_table        [n] int32, logical page -> physical page; entries must be
 *                     distinct and in [0, num_phys_pages) (precondition, not checked
 *                     on the device)
 *   LSE               [Hq][C] float, natural log of the sum of exp(scaled logits)
 *   selection lists   [Hkv][sel_stride] int32 LOGICAL page ids, ascending, distinct,
 *                     with sel_count[g] valid entries; they must contain the m local
 *                     pages n_past..n-1 (so that no query row is empty)
 * All base pointers and strides must keep 16-byte alignment of every D-row.
 *
 * Errors: every entry point validates host-visible scalars and pointers before
 * anything is launched and returns a status; on any status other than OOMB_OK
 * nothing was enqueued.  OOMB_ERR_LAUNCH reports a failed kernel launch.
 */
#ifndef OOMB_H_
#define OOMB_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  OOMB_OK = 0,
  OOMB_ERR_INVALID_ARG = 1, /* NULL pointer, non-divisible sizes, bad stride/alignment */
  OOMB_ERR_UNSUPPORTED = 2, /* shape / dtype combination with no kernel */
  OOMB_ERR_WORKSPACE = 3,   /* workspace NULL or smaller than oomb_workspace_bytes() */
  OOMB_ERR_LAUNCH = 4,      /* HIP reported a launch error */
  OOMB_ERR_OUT_OF_PAGES = 5, /* oomb_page_pool_alloc: fewer free pages than asked for */
  OOMB_ERR_SCRATCH_LIMIT = 6 /* oomb_page_score_topk_noalloc: the shape needs more than the built-in scratch */
} oomb_status;

typedef enum { OOMB_F32 = 0, OOMB_BF16 = 1 } oomb_dtype;

typedef enum {
  OOMB_OP_SCORE_TOPK = 0,
  OOMB_OP_ATTN_FWD = 1,
  OOMB_OP_ATTN_BWD = 2,
  OOMB_OP_VOTE_TOPK = 3,   /* oomb_page_vote_topk */
  OOMB_OP_ATTN_FWD_QP = 4, /* oomb_paged_attn_fwd_qp */
  OOMB_OP_ATTN_BWD_QP = 5, /* oomb_paged_attn_bwd_qp */
  OOMB_OP_CHECK_INPUTS = 6 /* oomb_check_inputs */
} oomb_op;

typedef struct {
  int32_t n_q_heads;   /* Hq */
  int32_t n_kv_heads;  /* Hkv, divides Hq */
  int32_t head_dim;    /* D: 64 or 128 */
  int32_t page_size;   /* P: power of two, 16..128 */
  int32_t chunk_len;   /* C, multiple of P */
  int32_t dtype;       /* oomb_dtype of Q, K, V, O, dO, dQ */
  int32_t grad_dtype;  /* oomb_dtype of the dK / dV pools */
  float sm_scale;      /* logits = sm_scale * <q, k>; > 0 */
  int64_t ctx_len;     /* N, includes the chunk; multiple of P; N >= C */
  int64_t pool_page_stride, pool_head_stride, pool_tok_stride; /* elements */
  int64_t q_tok_stride, q_head_stride;                         /* elements */
  int64_t num_phys_pages; /* pages in each pool; n <= num_phys_pages */
} oomb_attn_desc;

/* Bytes of device workspace `op` needs for this descriptor.  top_k: for
 * OOMB_OP_SCORE_TOPK and OOMB_OP_VOTE_TOPK the number of pages to retrieve; for
 * OOMB_OP_ATTN_FWD and OOMB_OP_ATTN_BWD the selection list's row stride minus the m
 * local pages (i.e. the top_k the list was built with), or a negative value for a
 * dense call (sel_pages == NULL); for the _QP operations the lists' row stride minus
 * m (>= 0).  The _QP sizes cover the worst case in which the lists of a KV head share
 * no page (m * (top_k + m) distinct pages).  Returns 0 for an invalid descriptor. */
size_t oomb_workspace_bytes(const oomb_attn_desc* desc, int32_t top_k, int32_t op);

/*
 * Page scoring + top-k page selection (Sec. 4.2: each key page is represented
 * by the mean of its keys; the chunk's queries are aggregated into one score
 * per key page; the top-K pages are kept).  Per KV head g:
 *   qbar[g]     = mean over the C tokens and the G heads of group g of Q
 *   kbar[g][l]  = mean of the P keys of logical page l (read through page_table)
 *   score[g][l] = <qbar[g], kbar[g][l]>              for past pages l < n_past
 * in IEEE binary32 with a fixed operation order (no fused multiply-add):
 * token sums run left to right, qbar sums query pages (outer) then heads
 * (inner), the dot product is a stride-halving tree over d.  The k_eff =
 * min(top_k, n_past) past pages with the largest score are kept, ties going to
 * the lower logical id (-0 == +0); the m local pages are appended; the list is
 * written in ascending logical id.  Scores must be finite.
 *
 *   q          [C][Hq][D]                        in
 *   k_pool     K pool                            in
 *   page_table [n]                               in
 *   sel_pages  [Hkv][top_k + m] int32            out (entries past sel_count[g] = -1)
 *   sel_count  [Hkv] int32                       out
 *   scores_out [Hkv][n_past] float or NULL       out
 * top_k >= 0.  Returns OOMB_ERR_UNSUPPORTED when n_past exceeds 1,048,576.
 */
oomb_status oomb_page_score_topk(const oomb_attn_desc* desc, const void* q, const void* k_pool,
                                 const int32_t* page_table, int32_t top_k, int32_t* sel_pages,
                                 int32_t* sel_count, float* scores_out, void* workspace,
                                 size_t workspace_bytes, void* hip_stream);

/*
 * oomb_page_score_topk for callers that cannot allocate or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the
 * workspace, same kernels, same results bit for bit; the scoring scratch (query-page sums, pooled
 * queries and, when scores_out is NULL, the scores) lives in a static device array of
 * OOMB_NOALLOC_SCRATCH_BYTES that every device the library runs on holds until the process ends.
 * Nothing is allocated or freed, here or in any library the call reaches (the first call on a device
 * looks the array's address up once).  A shape whose oomb_workspace_bytes(desc, top_k,
 * OOMB_OP_SCORE_TOPK) exceeds OOMB_NOALLOC_SCRATCH_BYTES is refused with OOMB_ERR_SCRATCH_LIMIT before
 * anything is launched (Hq * m * D + Hkv * (D + n_past) floats: the 4M-token benchmark shape needs
 * 1.4 MiB).  All calls on one device share the one array, which keeps the last call's contents (no
 * part of it has to start at zero): calls that overlap on a device -- two streams, two threads --
 * race; serialise them.
 */
#define OOMB_NOALLOC_SCRATCH_BYTES (4u << 20)
oomb_status oomb_page_score_topk_noalloc(const oomb_attn_desc* desc, const void* q, const void* k_pool,
                                         const int32_t* page_table, int32_t top_k, int32_t* sel_pages,
                                         int32_t* sel_count, float* scores_out, void* hip_stream);

/*
 * Paged attention forward (Sec. 4.1 operator over the pages of Sec. 4.2).
 * For every query head h and chunk row i:
 *   s_t = sm_scale * <Q[i,h], K[t,g]> over the visible tokens t,
 *   LSE[h][i] = log sum_t exp(s_t),  O[i,h,:] = sum_t exp(s_t - LSE) V[t,g,:].
 *   sel_pages == NULL selects every logical page 0..n-1 (dense); then sel_count
 *   and sel_stride are ignored.
 *   o   [C][Hq][D] out (overwritten);  lse [Hq][C] float out (overwritten).
 */
oomb_status oomb_paged_attn_fwd(const oomb_attn_desc* desc, const void* q, const void* k_pool,
                                const void* v_pool, const int32_t* page_table,
                                const int32_t* sel_pages, const int32_t* sel_count,
                                int32_t sel_stride, void* o, float* lse, void* workspace,
                                size_t workspace_bytes, void* hip_stream);

/*
 * Paged attention backward (Sec. 3 Eq. 3: KV gradients of earlier chunks
 * accumulate over later chunks' backward passes; Sec. 4.1: in-place
 * accumulation into the paged gradient pool; Sec. 4.2: the forward's page
 * indices are reused).  With p_t = exp(s_t - LSE), Delta = <dO[i,h], O[i,h]>,
 * dp_t = <dO[i,h], V[t,g]>, ds_t = p_t (dp_t - Delta):
 *   dQ[i,h,:]           = sm_scale * sum_t ds_t K[t,g,:]                (overwritten)
 *   dK pool[t,g,:]     += sm_scale * sum_{h in g} sum_i ds_t Q[i,h,:]    (accumulated)
 *   dV pool[t,g,:]     += sum_{h in g} sum_i p_t dO[i,h,:]               (accumulated)
 * at pool[page_table[t / P]][g][t % P][:], for the tokens of the selected pages
 * only; every other page of the gradient pools is left bit-identical.  The
 * pools are never zeroed here.  Each (KV head, page) is updated by exactly one
 * workgroup with plain loads and stores (no atomics), so results do not depend
 * on scheduling.  `sel_pages` must be the list the forward used; `o` and `lse`
 * are the forward's outputs.
 */
oomb_status oomb_paged_attn_bwd(const oomb_attn_desc* desc, const void* q, const void* k_pool,
                                const void* v_pool, const int32_t* page_table,
                                const int32_t* sel_pages, const int32_t* sel_count,
                                int32_t sel_stride, const void* o, const float* lse,
                                const void* d_o, void* d_q, void* dk_pool, void* dv_pool,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Retrieval by voting (Sec. 4.2, the scoring equation): per KV head g and query page tau,
 *   z[h][i][l]      = sm_scale * <Q[i,h], kbar[l][g]>          past pages l < n_past
 *   p[h][i][.]      = softmax of z[h][i][.] over the past pages l
 *   vote[g][tau][l] = sum of p[h][i][l] over the G heads h of group g and the P tokens i of query page tau
 * and the k_eff = min(top_k, n_past) past pages with the largest vote are kept (ties to the
 * lower logical id), followed by the local pages n_past .. n_past + tau that the rows of the
 * query page can see; lists ascending.  kbar is the page mean as kept by oomb_kv_append /
 * oomb_page_means; for bf16 tensors it is rounded to bf16 (nearest even) before the products,
 * which run on bf16 matrix instructions with fp32 accumulation; softmax and vote sums are fp32,
 * in a fixed order (results are bit-reproducible, but not bit-equal to another summation order).
 *   q          [C][Hq][D]                         in
 *   kbar_cache [>= n_past][Hkv][D] float          in
 *   sel_pages  [Hkv][m][top_k + m] int32          out (unused tail = -1)
 *   sel_count  [Hkv][m] int32                     out
 *   votes_out  [Hkv][m][n_past] float or NULL     out
 * Workspace: oomb_workspace_bytes(desc, top_k, OOMB_OP_VOTE_TOPK).  Returns
 * OOMB_ERR_UNSUPPORTED when n_past exceeds 1,048,576 or Hkv * m exceeds 65,535.
 */
oomb_status oomb_page_vote_topk(const oomb_attn_desc* desc, const void* q, const float* kbar_cache, int32_t top_k,
                                int32_t* sel_pages, int32_t* sel_count, float* votes_out, void* workspace,
                                size_t workspace_bytes, void* hip_stream);

/*
 * Attention with one page list per (KV head, query page) (Sec. 4.2: the votes are
 * aggregated for each of the m query pages of the chunk, so every query page
 * retrieves its own top-K key pages).  Same operators as oomb_paged_attn_fwd / _bwd,
 * except that chunk row i of a head of KV head g sees token t iff t <= a_i and page
 * t / P is in the list of (g, query page i / P):
 *   sel_pages [Hkv][m][sel_stride] int32 logical page ids, ascending, distinct, in [0, n)
 *   sel_count [Hkv][m]             valid entries of each list
 * The list of query page tau must hold the local page n_past + tau (so that no row is
 * empty); local pages beyond it may be listed and are ignored.  sel_stride >= m.
 * dK / dV: every page that appears in some list of KV head g is updated by exactly one
 * workgroup per slice of the query pages that list it, slices being added in a fixed
 * order (no atomics on results; bit-reproducible); pages in no list are untouched.
 * Workspace: oomb_workspace_bytes(desc, sel_stride - m, OOMB_OP_ATTN_FWD_QP / _BWD_QP).
 */
oomb_status oomb_paged_attn_fwd_qp(const oomb_attn_desc* desc, const void* q, const void* k_pool,
                                   const void* v_pool, const int32_t* page_table,
                                   const int32_t* sel_pages, const int32_t* sel_count,
                                   int32_t sel_stride, void* o, float* lse, void* workspace,
                                   size_t workspace_bytes, void* hip_stream);
oomb_status oomb_paged_attn_bwd_qp(const oomb_attn_desc* desc, const void* q, const void* k_pool,
                                   const void* v_pool, const int32_t* page_table,
                                   const int32_t* sel_pages, const int32_t* sel_count,
                                   int32_t sel_stride, const void* o, const float* lse,
                                   const void* d_o, void* d_q, void* dk_pool, void* dv_pool,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Paged-manager steps either side of the attention path (Sec. 4.1: the KV cache
 * grows chunk by chunk in pages).
 *
 * oomb_kv_append: the chunk's keys and values become its m = C/P local pages.
 *   k_chunk, v_chunk [C][Hkv][D] contiguous, device, in   (token order, desc->dtype)
 *   page_table[n]    device, in: entries n_past .. n-1 name the pages to fill
 *   k_pool, v_pool   device, in/out: token i of the chunk is copied, bit for bit, to
 *                    pool[page_table[n_past + i / P]][g][i % P][:]; nothing else is written
 *   kbar_cache       device, [>= n][Hkv][D] float, may be NULL: rows n_past .. n-1
 *                    receive the means of the new pages, k_bar = (sum of the P keys,
 *                    left to right) * (1/P) in binary32 -- the page representative of
 *                    Sec. 4.2, in the operation order of oomb_page_score_topk.
 * oomb_page_means: the same means for logical pages first_page .. first_page + n_pages - 1
 *   (0 <= first_page, first_page + n_pages <= n), e.g. to build the cache of a pool
 *   that was filled by other means.
 * oomb_page_score_topk_cached: oomb_page_score_topk with k_bar read from kbar_cache
 *   (rows 0 .. n_past-1) instead of being recomputed from the keys; same scores, bit
 *   for bit, same lists; reads n_past * Hkv * D floats instead of every past key.
 *   Workspace as for OOMB_OP_SCORE_TOPK.
 * oomb_local_page_list (Sec. 4.2, natively sparse models: local-attention layers
 *   retrieve only the most recent pages): for every KV head the min(window_pages,
 *   n_past) most recent past pages followed by the m local pages, ascending.
 *   sel_pages [Hkv][window_pages + m] (unused tail = -1), sel_count [Hkv].
 * Errors as for the other entry points (NULL / misaligned pointers, bad ranges:
 * OOMB_ERR_INVALID_ARG; nothing is launched).
 */
oomb_status oomb_kv_append(const oomb_attn_desc* desc, const void* k_chunk, const void* v_chunk,
                           const int32_t* page_table, void* k_pool, void* v_pool, float* kbar_cache,
                           void* hip_stream);
oomb_status oomb_page_means(const oomb_attn_desc* desc, const void* k_pool, const int32_t* page_table,
                            int64_t first_page, int64_t n_pages, float* kbar_cache, void* hip_stream);
oomb_status oomb_page_score_topk_cached(const oomb_attn_desc* desc, const void* q, const float* kbar_cache,
                                        int32_t top_k, int32_t* sel_pages, int32_t* sel_count,
                                        float* scores_out, void* workspace, size_t workspace_bytes,
                                        void* hip_stream);
oomb_status oomb_local_page_list(const oomb_attn_desc* desc, int32_t window_pages, int32_t* sel_pages,
                                 int32_t* sel_count, void* hip_stream);

/*
 * Page bookkeeping of the paged memory manager (Sec. 4.1: the KV cache and its gradients
 * live in fixed-size pages handed out on demand, so a growing context never reallocates
 * or fragments memory).  The K, V, dK and dV pools share one page numbering, so one
 * free list serves all four.  HOST-side and stateless: the caller owns
 *     free_stack [num_phys_pages] int32, host   the free physical pages (a stack)
 *     n_free     int64, host                    how many of its leading entries are valid
 * and builds the page table from the pages it is given (entries n_past .. n-1 of
 * `page_table` for oomb_kv_append).  Deterministic: after a reset pages come out in
 * ascending order 0, 1, 2, ...; released pages are reused last-released-first.
 *   oomb_page_pool_reset    every page free.
 *   oomb_page_pool_alloc    pops `count` pages into pages_out[count]; if fewer are free nothing
 *                           changes and OOMB_ERR_OUT_OF_PAGES is returned (the pools are full).
 *   oomb_page_pool_release  pushes pages[count] back (in the order given).  A page out of range, listed
 *                           twice or already free: OOMB_ERR_INVALID_ARG, nothing changes
 *                           (checked against the whole stack: O(count * n_free)).
 * NULL pointers and negative counts: OOMB_ERR_INVALID_ARG.  No device work, no stream.
 */
oomb_status oomb_page_pool_reset(int64_t num_phys_pages, int32_t* free_stack, int64_t* n_free);
oomb_status oomb_page_pool_alloc(int32_t* free_stack, int64_t* n_free, int64_t count, int32_t* pages_out);
oomb_status oomb_page_pool_release(int64_t num_phys_pages, int32_t* free_stack, int64_t* n_free,
                                   const int32_t* pages, int64_t count);

/*
 * Offloaded KV cache (Sec. 4.3: the KV cache and its gradients are kept in host memory, the
 * pages a chunk needs are transferred asynchronously; pinned memory and dedicated streams).
 * The host pools are PINNED HOST memory that the device can address (hipHostMalloc, or a
 * pinned torch tensor); they have the layout and strides of the descriptor's pools.  The
 * transfers are kernels that read / write that memory directly, one (page, KV head) tile
 * after the other on a few workgroups, enqueued on hip_stream like everything else: put them
 * on a stream of their own to overlap them with computation, and order them against the
 * attention calls with events.
 *
 * oomb_offload_plan: which pages the lists hold, and a staging slot for each.
 *     sel_pages / sel_count: lists_per_head = 1: [Hkv][sel_stride] / [Hkv] (oomb_page_score_topk*);
 *                            lists_per_head = m: [Hkv][m][sel_stride] / [Hkv][m] (oomb_page_vote_topk)
 *     stage_capacity  pages in each staging pool (> 0)
 *     head_mask   [n] uint32 device, out: bit g set iff some list of KV head g holds the page
 *     stage_table [n] int32 device, out: THE PAGE TABLE OF THE STAGING POOLS -- the slot of a held page,
 *                 slots numbered in ascending logical page order over all held pages; -1 for a page in no
 *                 list (the attention kernels look up listed pages only).  It never points outside the
 *                 staging pools: a held page whose slot would be >= stage_capacity gets slot 0.
 *     slot_pages  [stage_capacity] int32 device, out: page of every slot in use
 *     n_slots     [2] int32 device, out: [0] slots in use = min(pages held, stage_capacity),
 *                 [1] pages held.  n_slots[1] > stage_capacity means the staging pools are too small:
 *                 fetch and write-back then move the first stage_capacity pages only and attention over
 *                 the staging pools, while it stays inside them, returns meaningless values -- check
 *                 n_slots[1] (it is device memory: with the next host synchronisation) before trusting a
 *                 step.  min(n, Hkv * lists_per_head * sel_stride) slots always suffice.
 *   Hkv <= 32 (else OOMB_ERR_UNSUPPORTED).
 * oomb_offload_fetch: for every slot s < n_slots[0] (and < stage_capacity), l = slot_pages[s], and every
 *   KV head g with bit g of head_mask[l] set,
 *     stage_k / stage_v [s][g][:][:] = host_k / host_v [page_table[l]][g][:][:]
 *   bit for bit; if stage_dk / stage_dv are given (both or neither) the same tiles of the
 *   gradient staging pools are zeroed.  Staging pools: device memory, descriptor strides,
 *   stage_capacity pages; the other tiles of a slot are left alone and are never read by the
 *   attention kernels.  The attention entry points then run on the staging pools with
 *   page_table = stage_table (their descriptor keeps num_phys_pages >= n: the bound is on the
 *   table's domain).
 * oomb_offload_writeback: for the same (s, g),
 *     host_dk / host_dv [page_table[l]][g] += stage_dk / stage_dv [s][g]
 *   in float (rounded to the pool's dtype for bf16 pools); nothing else is written.
 * Errors: OOMB_ERR_INVALID_ARG also for a host pool that is not device-addressable memory
 * (checked with hipPointerGetAttributes before anything is launched).
 */
oomb_status oomb_offload_plan(const oomb_attn_desc* desc, const int32_t* sel_pages, const int32_t* sel_count,
                              int32_t sel_stride, int32_t lists_per_head, int32_t stage_capacity, int32_t* stage_table,
                              int32_t* slot_pages, uint32_t* head_mask, int32_t* n_slots, void* hip_stream);
oomb_status oomb_offload_fetch(const oomb_attn_desc* desc, const void* host_k_pool, const void* host_v_pool,
                               const int32_t* page_table, const int32_t* slot_pages, const uint32_t* head_mask,
                               const int32_t* n_slots, int32_t stage_capacity, void* stage_k, void* stage_v,
                               void* stage_dk, void* stage_dv, void* hip_stream);
oomb_status oomb_offload_writeback(const oomb_attn_desc* desc, const void* stage_dk, const void* stage_dv,
                                   void* host_dk_pool, void* host_dv_pool, const int32_t* page_table,
                                   const int32_t* slot_pages, const uint32_t* head_mask, const int32_t* n_slots,
                                   int32_t stage_capacity, void* hip_stream);

/*
 * Debug aid: the documented preconditions of the attention entry points, checked on the device
 * (the hot path trusts them).  Writes a bit mask to violations[0] (device, int32):
 *   1  a page_table entry (logical pages 0 .. n-1) outside [0, num_phys_pages)
 *   2  two logical pages mapped to the same physical page
 *   4  a list count outside [0, sel_stride]
 *   8  a list entry outside [0, n)
 *   16 a list that is not strictly ascending (this also catches duplicates)
 *   32 a list without the local pages it must hold: all m of them for lists_per_head = 1
 *      ([Hkv][sel_stride]), page n_past + tau for the list of query page tau with
 *      lists_per_head = m ([Hkv][m][sel_stride])
 * sel_pages == NULL checks the page table only.  One workgroup; reads only, apart from the
 * workspace (oomb_workspace_bytes(desc, 0, OOMB_OP_CHECK_INPUTS) = num_phys_pages int32) and
 * violations[0].  No index is dereferenced before it has been checked.
 */
oomb_status oomb_check_inputs(const oomb_attn_desc* desc, const int32_t* page_table, const int32_t* sel_pages,
                              const int32_t* sel_count, int32_t sel_stride, int32_t lists_per_head, int32_t* violations,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

const char* oomb_status_string(int32_t status);

/* major * 10000 + minor * 100 + patch */
int32_t oomb_version(void);

#ifdef __cplusplus
}
#endif
#endif /* OOMB_H_ */
