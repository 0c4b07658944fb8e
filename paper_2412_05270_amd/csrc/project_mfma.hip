// Matrix-core projection R = P G for bf16 gradients (Algorithm 1, step 1).
#include "apollo_internal.h"

namespace apollo {

bool project_mfma_supported(int rows, int cols, bool left, bool bf16, int r) {
  (void)rows; (void)cols; (void)left; (void)bf16; (void)r;
  return false;
}

hipError_t launch_project_mfma(const TensorDesc* d_descs, int count, int rows, int cols, bool left,
                               const StepParams& sp, hipStream_t st) {
  (void)d_descs; (void)count; (void)rows; (void)cols; (void)left; (void)sp; (void)st;
  return hipErrorNotSupported;
}

}  // namespace apollo
