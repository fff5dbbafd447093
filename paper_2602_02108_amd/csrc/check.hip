// Debug aid: the preconditions of the attention entry points, checked on the device (paper
// Sec. 4.1: the page table maps logical pages to distinct physical pages; Sec. 4.2: the lists
// hold retrieved pages plus the chunk's own pages).  The hot path trusts them; this kernel reads
// the same arrays, never dereferences an unchecked index, and reports a bit mask of violations.
#include "common.h"
#include "launch.h"

namespace oomb {

constexpr int CHK_THREADS = 1024;
enum {
  CHK_TABLE_RANGE = 1, CHK_TABLE_DISTINCT = 2, CHK_LIST_COUNT = 4, CHK_LIST_RANGE = 8, CHK_LIST_ORDER = 16,
  CHK_LIST_LOCAL = 32
};

// One workgroup.  marks: [num_phys] int32 scratch.  lists_per_head: 0 = no lists, 1, or m.
__global__ __launch_bounds__(CHK_THREADS) void check_inputs_kernel(Params p, int64_t num_phys, int32_t lists_per_head,
                                                                  int32_t* __restrict__ marks, int32_t* __restrict__ out) {
  __shared__ int32_t bad_s;
  const int tid = threadIdx.x;
  if (tid == 0) bad_s = 0;
  for (int64_t q = tid; q < num_phys; q += CHK_THREADS) marks[q] = 0;
  __syncthreads();
  int32_t bad = 0;
  const int32_t n = (int32_t)p.n;
  for (int32_t l = tid; l < n; l += CHK_THREADS) {
    const int32_t q = p.page_table[l];
    if (q < 0 || q >= num_phys) bad |= CHK_TABLE_RANGE;
    else if (atomicAdd(&marks[q], 1) > 0) bad |= CHK_TABLE_DISTINCT;  // (whoever comes second reports)
  }
  if (lists_per_head > 0) {
    const int32_t n_lists = p.Hkv * lists_per_head;
    for (int32_t li = 0; li < n_lists; ++li) {
      const int32_t* lst = p.sel + (int64_t)li * p.sel_stride;
      int32_t c = p.sel_count[li];
      if (c < 0 || c > p.sel_stride) {
        bad |= CHK_LIST_COUNT;
        c = c < 0 ? 0 : p.sel_stride;
      }
      // local pages this list must hold: all m of them, or the one of its query page
      const int32_t need_lo = lists_per_head == 1 ? (int32_t)p.n_past : (int32_t)p.n_past + li % lists_per_head;
      const int32_t need_hi = lists_per_head == 1 ? n - 1 : need_lo;
      int32_t found = 0;
      for (int32_t j = tid; j < c; j += CHK_THREADS) {
        const int32_t e = lst[j];
        if (e < 0 || e >= n) bad |= CHK_LIST_RANGE;
        if (j > 0 && lst[j - 1] >= e) bad |= CHK_LIST_ORDER;
        found += e >= need_lo && e <= need_hi;
      }
      // the required local pages are need_hi - need_lo + 1 distinct values: count them over the workgroup
      // (with duplicates the order bit is raised anyway)
      __shared__ int32_t found_s;
      if (tid == 0) found_s = 0;
      __syncthreads();
      if (found) atomicAdd(&found_s, found);
      __syncthreads();
      if (tid == 0 && found_s < need_hi - need_lo + 1) bad |= CHK_LIST_LOCAL;
      __syncthreads();
    }
  }
  if (bad) atomicOr(&bad_s, bad);
  __syncthreads();
  if (tid == 0) out[0] = bad_s;
}

hipError_t launch_check_inputs(const Params& p, int64_t num_phys, int32_t lists_per_head, int32_t* marks, int32_t* out,
                               hipStream_t st) {
  check_inputs_kernel<<<dim3(1), dim3(CHK_THREADS), 0, st>>>(p, num_phys, lists_per_head, marks, out);
  return hipGetLastError();
}

}  // namespace oomb
