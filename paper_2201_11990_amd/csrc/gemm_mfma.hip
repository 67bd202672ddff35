// bf16 MFMA GEMM (placeholder until the kernel lands): reports every problem as
// unsupported so the dispatcher takes the vector-ALU kernel.
#include "common.h"
namespace mtnlg {
int gemm_mfma_bf16(int, int64_t, int64_t, int64_t, const void *, const void *, void *, const void *, void *,
                   uint32_t, hipStream_t) {
  return MTNLG_UNSUPPORTED_SHAPE;
}
}  // namespace mtnlg
