// Backward bf16 MFMA kernels (placeholder until they land).
#include "common.h"

namespace oomb {
hipError_t launch_bwd_generic(const Params& p, bool is_bf16, int32_t max_list_len, hipStream_t st);
hipError_t launch_bwd_mfma(const Params& p, int32_t max_list_len, void*, hipStream_t st) {
  return launch_bwd_generic(p, true, max_list_len, st);
}
size_t bwd_mfma_workspace_bytes(const Params&, int32_t) { return 0; }
}  // namespace oomb
