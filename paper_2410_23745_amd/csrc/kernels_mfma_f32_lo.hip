// Instantiations of the MFMA contraction kernel: fp32 tile variants 0-3.
#include "conv_mfma.h"

namespace syno {

void launch_mfma_f32_lo(int vi, const MfmaParams& p, const void* X, const void* W, void* out, hipStream_t s) {
#define SYNO_CASE(VI)                                              \
  case VI:                                                         \
    if (p.U == 3) launch_variant<false, VI, 3, 0, false>(p, X, W, out, s); \
    else launch_variant<false, VI, 1, 0, false>(p, X, W, out, s);     \
    break;
  switch (vi) {
    SYNO_CASE(0) SYNO_CASE(1) SYNO_CASE(2) SYNO_CASE(3)
    default: break;
  }
#undef SYNO_CASE
}

}  // namespace syno
