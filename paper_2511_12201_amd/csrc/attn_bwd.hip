// Backward of the sparse attention (placeholder until the kernels land).
#include "common.h"
#include "kernels.h"

namespace omni {

size_t attn_bwd_ws(const Layer&, int, int) { return 256; }

int run_attn_bwd(const Layer&, int, const void*, const void*, const void*, const void*, const void*, const float*,
                 const int*, const int*, const int*, const int*, int, void*, void*, void*, void*, hipStream_t) {
  OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "omni_sparse_attn_bwd is not implemented yet");
}

}  // namespace omni
