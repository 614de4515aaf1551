// Instantiations of the MFMA contraction kernel: bf16 tile variants 0, 2-5, 7 and 10, fp32 result (the others
// live in kernels_mfma_bf16_f32out_b.hip, so that the two halves compile side by side).
#include "conv_mfma.h"

namespace syno {

void launch_mfma_bf16_f32out_b(int vi, const MfmaParams& p, const void* X, const void* W, void* out, hipStream_t s);

void launch_mfma_bf16_f32out(int vi, const MfmaParams& p, const void* X, const void* W, void* out, hipStream_t s) {
#define SYNO_CASE(VI)                                                 \
  case VI:                                                            \
    if (p.wf == 9) launch_variant<true, VI, 1, 9, false>(p, X, W, out, s); \
    else launch_variant<true, VI, 1, 0, false>(p, X, W, out, s);       \
    break;
  switch (vi) {
    SYNO_CASE(2) SYNO_CASE(3) SYNO_CASE(4) SYNO_CASE(5) SYNO_CASE(7)
    case 0:   // also reads forward-layout weights of 3-tap windows itself
      if (p.wf == 9) launch_variant<true, 0, 1, 9, false>(p, X, W, out, s);
      else if (p.wf == 3) launch_variant<true, 0, 1, 3, false>(p, X, W, out, s);
      else launch_variant<true, 0, 1, 0, false>(p, X, W, out, s);
      break;
    case 10:  // 1x1 windows only: packed weights
      launch_variant<true, 10, 1, 0, false>(p, X, W, out, s);
      break;
    case 1: case 6: case 8: case 9:
      launch_mfma_bf16_f32out_b(vi, p, X, W, out, s);
      break;
    default: break;
  }
#undef SYNO_CASE
}

}  // namespace syno
