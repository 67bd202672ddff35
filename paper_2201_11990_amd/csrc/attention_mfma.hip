// bf16 MFMA attention (placeholder until the kernels land).
#include "common.h"
namespace mtnlg {
bool attention_mfma_supported(int, int) { return false; }
size_t attention_bwd_workspace_bytes(int b, int s, int n, int) { return (size_t)b * n * s * sizeof(float); }
int attention_fwd_mfma(int, int, int, int, float, const void *, void *, float *, hipStream_t) {
  return MTNLG_UNSUPPORTED_SHAPE;
}
int attention_bwd_mfma(int, int, int, int, float, const void *, const void *, const float *, const void *,
                       void *, void *, hipStream_t) {
  return MTNLG_UNSUPPORTED_SHAPE;
}
}  // namespace mtnlg
