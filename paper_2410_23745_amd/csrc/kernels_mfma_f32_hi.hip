// Instantiations of the MFMA contraction kernel: fp32 tile variants 4-13.
#include "conv_mfma.h"

namespace syno {

void launch_mfma_f32_hi(int vi, const MfmaParams& p, const void* X, const void* W, void* out, hipStream_t s) {
#define SYNO_CASE(VI)                                              \
  case VI:                                                         \
    if (p.U == 3) launch_variant<false, VI, 3, 0, false>(p, X, W, out, s); \
    else launch_variant<false, VI, 1, 0, false>(p, X, W, out, s);     \
    break;
  switch (vi) {
    SYNO_CASE(4) SYNO_CASE(5) SYNO_CASE(6) SYNO_CASE(7) SYNO_CASE(8) SYNO_CASE(9) SYNO_CASE(10) SYNO_CASE(11) SYNO_CASE(12) SYNO_CASE(13)
    default: break;
  }
#undef SYNO_CASE
}

}  // namespace syno
