// bf16 MFMA kernels of the scoring stage (placeholder translation unit: the
// ALU kernels in score.hip serve every layer shape until these are enabled).
#include "score_common.h"

namespace ifkv {

bool score_mfma_supported(const ifkv_ctx *, int) { return false; }

hipError_t launch_score_mfma(ifkv_ctx *, const void *, int64_t, const void *, int, const void *, int, float *) {
  return hipErrorNotSupported;
}

}  // namespace ifkv
