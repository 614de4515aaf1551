// Instantiations of the MFMA contraction kernel: bf16 tile variants 1, 6, 8 and 9, fp32 result.
#include "conv_mfma.h"

namespace syno {

void launch_mfma_bf16_f32out_b(int vi, const MfmaParams& p, const void* X, const void* W, void* out, hipStream_t s) {
#define SYNO_CASE_ADJ(VI)   /* also instantiated for backward-data straight from forward-layout 3x3 weights */ \
  case VI:                                                            \
    if (p.wf == 9) launch_variant<true, VI, 1, 9, false>(p, X, W, out, s); \
    else if (p.wf == -9) launch_variant<true, VI, 1, -9, false>(p, X, W, out, s); \
    else launch_variant<true, VI, 1, 0, false>(p, X, W, out, s);       \
    break;
  switch (vi) {
    SYNO_CASE_ADJ(1) SYNO_CASE_ADJ(8) SYNO_CASE_ADJ(9)
    case 6:   // single chunk: packed weights, or weights as they lie in memory with 1, 3 or 9 taps per channel (negative: backward-data)
      if (p.wf == 9) launch_variant<true, 6, 1, 9, false>(p, X, W, out, s);
      else if (p.wf == 3) launch_variant<true, 6, 1, 3, false>(p, X, W, out, s);
      else if (p.wf == 1) launch_variant<true, 6, 1, 1, false>(p, X, W, out, s);
      else if (p.wf == -9) launch_variant<true, 6, 1, -9, false>(p, X, W, out, s);
      else if (p.wf == -3) launch_variant<true, 6, 1, -3, false>(p, X, W, out, s);
      else if (p.wf == -1) launch_variant<true, 6, 1, -1, false>(p, X, W, out, s);
      else launch_variant<true, 6, 1, 0, false>(p, X, W, out, s);
      break;
    default: break;
  }
#undef SYNO_CASE_ADJ
}

}  // namespace syno
