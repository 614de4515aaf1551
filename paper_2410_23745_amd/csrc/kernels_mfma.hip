// MFMA contraction family (placeholder until the tuned kernels land).
#include <hip/hip_runtime.h>

#include "plan.h"

namespace syno {
syno_status launch_mfma(const syno_plan*, int, const void*, const void*, void*, void*, hipStream_t) {
  return SYNO_ERR_UNSUPPORTED;
}
}  // namespace syno
