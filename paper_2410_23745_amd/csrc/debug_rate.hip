// Measurement aid: a kernel that does nothing but issue MFMAs, so that a benchmark can print the matrix-core rate
// this device actually sustains next to the datasheet peak.  Not on any operator's path.
#include <hip/hip_runtime.h>

#include "syno.h"

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
constexpr int kAcc = 16;      // independent accumulators per wave: enough to cover the MFMA latency

template <bool BF>
__global__ __launch_bounds__(256) void mfma_rate(float* out, int iters) {
  floatx4 acc[kAcc];
#pragma unroll
  for (int i = 0; i < kAcc; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
  const float seed = threadIdx.x * 1e-3f;
  bf16x8 a8, b8;
#pragma unroll
  for (int i = 0; i < 8; ++i) { a8[i] = (__bf16)seed; b8[i] = (__bf16)1.0f; }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kAcc; ++i) {
      if constexpr (BF) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, b8, acc[i], 0, 0, 0);
      else acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(seed, 1.0f, acc[i], 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kAcc; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

extern "C" syno_status syno_debug_mfma_rate(syno_dtype dtype, int32_t iters, int32_t workgroups, float* out,
                                            int64_t* flop, hipStream_t stream) {
  if (!out || !flop) return SYNO_ERR_NULL;
  if (iters < 1 || workgroups < 1 || workgroups > 65536) return SYNO_ERR_SHAPE;
  // 4 waves per workgroup; one 16x16 MFMA is 2*16*16*K flop with K = 32 (bf16) or 4 (fp32)
  *flop = (int64_t)workgroups * 4 * iters * kAcc * 2 * 16 * 16 * (dtype == SYNO_BF16 ? 32 : 4);
  if (dtype == SYNO_BF16) hipLaunchKernelGGL(mfma_rate<true>, dim3(workgroups), dim3(256), 0, stream, out, iters);
  else hipLaunchKernelGGL(mfma_rate<false>, dim3(workgroups), dim3(256), 0, stream, out, iters);
  return hipGetLastError() == hipSuccess ? SYNO_OK : SYNO_ERR_HIP;
}
