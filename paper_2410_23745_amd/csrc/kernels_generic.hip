// General kernels: evaluate a lowered index program per (target element, free point).
// They serve every valid pGraph in all three directions; the tuned families replace them
// where the planner recognises a convolution-like form.
#include <hip/hip_runtime.h>

#include "plan.h"

namespace syno {
namespace {

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round to nearest, ties to even (finite inputs; NaN keeps a quiet payload)
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <bool BF>
__device__ __forceinline__ float load_elem(const void* p, int off) {
  if constexpr (BF) return bf16_to_f32(reinterpret_cast<const uint16_t*>(p)[off]);
  else return reinterpret_cast<const float*>(p)[off];
}

template <bool BF>
__device__ __forceinline__ void store_elem(void* p, int64_t off, float v) {
  if constexpr (BF) reinterpret_cast<uint16_t*>(p)[off] = f32_to_bf16(v);
  else reinterpret_cast<float*>(p)[off] = v;
}

// n / d for 0 <= n < 2^31 and d >= 1 with the precomputed magic of plan.h (0 for d = 1).
__host__ __device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t d, uint32_t magic) {
  if (d < 2) return n;
#if defined(__HIP_DEVICE_COMPILE__)
  return __umulhi(n, magic) >> (31 - __clz((int)(d - 1)));
#else
  return (uint32_t)(((uint64_t)n * magic) >> 32) >> (31 - __builtin_clz(d - 1));
#endif
}

// (flat indices are below 2^31)
__host__ __device__ __forceinline__ void decode(const AxisRef* ax, int n, int64_t flat64, int* v) {
  uint32_t flat = (uint32_t)flat64;
  for (int i = n - 1; i >= 0; --i) {
    const uint32_t s = (uint32_t)ax[i].size;
    const uint32_t q = fast_div(flat, s, (uint32_t)ax[i].stride);
    v[ax[i].slot] = (int)(flat - q * s);
    flat = q;
  }
}

// Runs ops [lo, hi) on the slot file; returns false when a range or divisibility test fails.
__host__ __device__ __forceinline__ bool run_ops(const IndexProgram& P, int lo, int hi, int* v) {
  bool ok = true;
  for (int k = lo; k < hi; ++k) {
    const IndexOp o = P.ops[k];
    switch (o.kind) {
      // (once a range test has failed the slots hold meaningless values; unsigned arithmetic keeps wrap-around defined)
      case OP_MULADD: v[o.d0] = (int)((uint32_t)v[o.a] * (uint32_t)o.p0 + (uint32_t)v[o.b]); break;
      case OP_DIVMOD: {      // (operands are coordinates, 0 <= x < 2^31, whenever the term is still valid)
        const int x = v[o.a];
        const int q = (int)fast_div((uint32_t)x, (uint32_t)o.p0, (uint32_t)o.p1);
        v[o.d0] = q;
        v[o.d1] = (int)((uint32_t)x - (uint32_t)q * (uint32_t)o.p0);
        break;
      }
      case OP_SHIFT:
        if (o.p2 == 0) {       // constant offset, already reduced mod p0: one conditional subtraction
          const int x = (int)((uint32_t)v[o.a] + (uint32_t)o.p1);
          v[o.d0] = x >= o.p0 ? x - o.p0 : x;
        } else {
          v[o.d0] = (int)((uint32_t)v[o.a] + (uint32_t)o.p1 + (uint32_t)o.p2 * (uint32_t)v[o.b]) % o.p0;
        }
        break;
      case OP_ADDCHK: {
        const int t = (int)((uint32_t)v[o.a] + (uint32_t)o.p2 * (uint32_t)v[o.b] + (uint32_t)o.p1);
        ok = ok && ((unsigned)t < (unsigned)o.p0);
        v[o.d0] = t;
        break;
      }
      case OP_MUL: v[o.d0] = (int)((uint32_t)v[o.a] * (uint32_t)o.p0); break;
      case OP_DIVCHK: {
        const int x = v[o.a];
        const int q = (int)fast_div((uint32_t)x, (uint32_t)o.p0, (uint32_t)o.p1);
        ok = ok && x >= 0 && (int)((uint32_t)q * (uint32_t)o.p0) == x;
        v[o.d0] = q;
        break;
      }
    }
  }
  return ok;
}

__host__ __device__ __forceinline__ int dot(const AxisRef* ax, int n, const int* v) {
  uint32_t off = 0;
  for (int i = 0; i < n; ++i) off += (uint32_t)v[ax[i].slot] * (uint32_t)ax[i].stride;
  return (int)off;
}

// out[t] = sum over free points q of A[a(t,q)] * B[b(t,q)], fp32 accumulation in blocks of 64 terms.
// COOP: one workgroup per target, its 256 lanes stride over the free points.
template <bool INBF, bool OUTBF, bool COOP>
__global__ __launch_bounds__(256) void index_program_contract(const IndexProgram P, const void* __restrict__ A,
                                                              const void* __restrict__ B, void* __restrict__ out) {
  const int64_t t = COOP ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (!COOP && t >= P.n_target) return;
  int v[kMaxSlots];
  for (int i = 0; i < kMaxSlots; ++i) v[i] = 0;
  decode(P.tgt, P.n_tgt, t, v);
  const bool ok0 = run_ops(P, 0, P.n_ops0, v);
  float total = 0.f, part = 0.f;
  if (ok0) {
    int cnt = 0;
    for (int64_t q = COOP ? threadIdx.x : 0; q < P.n_free; q += COOP ? 256 : 1) {
      decode(P.fre, P.n_fre, q, v);
      if (run_ops(P, P.n_ops0, P.n_ops, v)) {
        const float a = load_elem<INBF>(A, dot(P.a, P.n_a, v));
        const float b = load_elem<INBF>(B, dot(P.b, P.n_b, v));
        part = fmaf(a, b, part);
      }
      if (++cnt == 64) { total += part; part = 0.f; cnt = 0; }
    }
  }
  total += part;
  if constexpr (COOP) {
    __shared__ float red[4];
    for (int s = 32; s > 0; s >>= 1) total += __shfl_down(total, s, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = total;
    __syncthreads();
    if (threadIdx.x == 0) store_elem<OUTBF>(out, t, (red[0] + red[1]) + (red[2] + red[3]));
  } else {
    store_elem<OUTBF>(out, t, total);
  }
}

__global__ __launch_bounds__(256) void index_program_map(const IndexProgram P, const int64_t* __restrict__ t_flat,
                                                         const int64_t* __restrict__ q_flat, int64_t n,
                                                         int32_t* __restrict__ a_off, int32_t* __restrict__ b_off) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  int v[kMaxSlots];
  for (int k = 0; k < kMaxSlots; ++k) v[k] = 0;
  const int64_t t = t_flat[i], q = q_flat[i];
  bool ok = t >= 0 && t < P.n_target && q >= 0 && q < P.n_free;
  if (ok) {
    decode(P.tgt, P.n_tgt, t, v);
    decode(P.fre, P.n_fre, q, v);
    ok = run_ops(P, 0, P.n_ops, v);
  }
  a_off[i] = ok ? dot(P.a, P.n_a, v) : -1;
  b_off[i] = ok ? dot(P.b, P.n_b, v) : -1;
}

template <bool INBF, bool OUTBF>
void launch_typed(const IndexProgram& P, bool coop, const void* A, const void* B, void* out, hipStream_t s) {
  if (coop)
    hipLaunchKernelGGL((index_program_contract<INBF, OUTBF, true>), dim3((unsigned)P.n_target), dim3(256), 0, s, P, A, B,
                       out);
  else
    hipLaunchKernelGGL((index_program_contract<INBF, OUTBF, false>), dim3((unsigned)((P.n_target + 255) / 256)),
                       dim3(256), 0, s, P, A, B, out);
}

}  // namespace

syno_status launch_generic(const syno_plan* p, int which, const void* A, const void* B, void* out, hipStream_t stream) {
  const IndexProgram& P = p->prog[which];
  if (P.n_target <= 0) return SYNO_OK;
  const bool inbf = p->in_dtype == SYNO_BF16;
  const bool outbf = which != SYNO_BWD_WEIGHT && p->out_dtype == SYNO_BF16;
  const bool coop = p->launch[which].coop != 0;
  if (inbf && outbf) launch_typed<true, true>(P, coop, A, B, out, stream);
  else if (inbf) launch_typed<true, false>(P, coop, A, B, out, stream);
  else if (outbf) launch_typed<false, true>(P, coop, A, B, out, stream);
  else launch_typed<false, false>(P, coop, A, B, out, stream);
  return hipGetLastError() == hipSuccess ? SYNO_OK : SYNO_ERR_HIP;
}

syno_status launch_debug_gather(const syno_plan* p, int which, const int64_t* t, const int64_t* q, int64_t n,
                                int32_t* a_off, int32_t* b_off, hipStream_t stream) {
  if (n <= 0) return SYNO_OK;
  hipLaunchKernelGGL(index_program_map, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p->prog[which], t, q, n,
                     a_off, b_off);
  return hipGetLastError() == hipSuccess ? SYNO_OK : SYNO_ERR_HIP;
}

// The same index program run on the host, for checking a plan where no GPU is present.
syno_status host_debug_gather(const syno_plan* p, int which, const int64_t* t_flat, const int64_t* q_flat, int64_t n,
                              int32_t* a_off, int32_t* b_off) {
  const IndexProgram& P = p->prog[which];
  for (int64_t i = 0; i < n; ++i) {
    int v[kMaxSlots] = {};
    const int64_t t = t_flat[i], q = q_flat[i];
    bool ok = t >= 0 && t < P.n_target && q >= 0 && q < P.n_free;
    if (ok) {
      decode(P.tgt, P.n_tgt, t, v);
      decode(P.fre, P.n_fre, q, v);
      ok = run_ops(P, 0, P.n_ops, v);
    }
    a_off[i] = ok ? dot(P.a, P.n_a, v) : -1;
    b_off[i] = ok ? dot(P.b, P.n_b, v) : -1;
  }
  return SYNO_OK;
}

}  // namespace syno
