// Page bookkeeping of the paged memory manager (paper Sec. 4.1): a free list of the
// physical pages that the K, V, dK and dV pools share.  Host code only; the state (a stack
// of free page ids and its fill level) belongs to the caller.
#include "common.h"

extern "C" {

oomb_status oomb_page_pool_reset(int64_t num_phys_pages, int32_t* free_stack, int64_t* n_free) {
  if (!free_stack || !n_free || num_phys_pages < 0 || num_phys_pages > INT32_MAX) return OOMB_ERR_INVALID_ARG;
  // the top of the stack is its last valid entry: page 0 comes out first
  for (int64_t i = 0; i < num_phys_pages; ++i) free_stack[i] = (int32_t)(num_phys_pages - 1 - i);
  *n_free = num_phys_pages;
  return OOMB_OK;
}

oomb_status oomb_page_pool_alloc(int32_t* free_stack, int64_t* n_free, int64_t count, int32_t* pages_out) {
  if (!free_stack || !n_free || count < 0 || (count > 0 && !pages_out) || *n_free < 0) return OOMB_ERR_INVALID_ARG;
  if (count > *n_free) return OOMB_ERR_OUT_OF_PAGES;
  for (int64_t i = 0; i < count; ++i) pages_out[i] = free_stack[*n_free - 1 - i];
  *n_free -= count;
  return OOMB_OK;
}

oomb_status oomb_page_pool_release(int64_t num_phys_pages, int32_t* free_stack, int64_t* n_free, const int32_t* pages,
                                   int64_t count) {
  if (!free_stack || !n_free || count < 0 || (count > 0 && !pages) || *n_free < 0 || *n_free > num_phys_pages)
    return OOMB_ERR_INVALID_ARG;
  if (count > num_phys_pages - *n_free) return OOMB_ERR_INVALID_ARG;  // more pages than are in use
  for (int64_t i = 0; i < count; ++i) {
    const int32_t pg = pages[i];
    if (pg < 0 || pg >= num_phys_pages) return OOMB_ERR_INVALID_ARG;
    for (int64_t j = 0; j < i; ++j)
      if (pages[j] == pg) return OOMB_ERR_INVALID_ARG;      // listed twice
    for (int64_t j = 0; j < *n_free; ++j)
      if (free_stack[j] == pg) return OOMB_ERR_INVALID_ARG;  // already free
  }
  for (int64_t i = 0; i < count; ++i) free_stack[*n_free + i] = pages[i];
  *n_free += count;
  return OOMB_OK;
}

}  // extern "C"
