// Bandwidth-bound family: per-channel (depthwise) window operators,
//   out[n,c,h,w] = sum_{kh,kw} W[c,kh,kw] * X[n,c,S*h+kh-ph,S*w+kw-pw]   (zero outside the plane),
// i.e. the convolution-like form with one input and one output channel per group.  About one
// flop per byte, so the kernel is a stream over X: every input element is fetched from HBM once,
// held in registers, and the window's horizontal neighbours come from the adjacent lanes of the
// wavefront through shuffles; no LDS.
//
// Work layout.  A "strip" is a run of RB output rows of one (n,c) plane.  A group of LPG lanes
// (a power of two) owns a strip; each lane owns V adjacent output columns and loads the S*V
// input columns under them as one vector per input row.  All S*RB+KH-S input rows of the strip
// are requested at once (one memory round trip), then the RB output rows are computed out of
// registers.  The input rows a strip shares with the strip above it are taken from the group above
// (same wave) with a shuffle instead of a second load.
#include <hip/hip_runtime.h>

#include <cstring>

#include <algorithm>

#include "plan.h"

namespace syno {
namespace {

struct DwParams {
  int32_t planes, C, Hi, Wi, Ho, Wo, ph, pw;
  int32_t lpg_log2;       // lanes per group = 1 << lpg_log2
  int32_t rb, strips;     // output rows per strip, strips per plane
  int32_t n_tasks;        // planes * strips
  int32_t ws_c, ws_kh, ws_kw;
  int32_t vec_ok;         // rows start 16-byte aligned and Wi is a multiple of S*V
};

// MODE 0: forward (B = weights, out = result).
// MODE 2: backward-weight partials: B = upstream gradient G (shaped like the forward result); every group
//         leaves the KH*KW sums of G[h][w] * window over its strip in out[task][KH*KW].
// Keeps the compiler from sinking a load below this point: everything requested so far is in flight together.
__device__ __forceinline__ void pin(float& v) { asm volatile("" : "+v"(v)); }

// VEC: rows start 16-byte aligned and hold a whole number of the lanes' vectors (one vector load per row).
template <int KH, int KW, int S, int V, int RB, int MODE, bool VEC>
__global__ __launch_bounds__(256) void depthwise_stream(const DwParams p, const float* __restrict__ X,
                                                        const float* __restrict__ Wt, float* __restrict__ out) {
  constexpr int SV = S * V;                      // input columns a lane loads per row
  constexpr int HL = KW / 2;                     // left neighbours needed (= pw)
  constexpr int HR = KW - KW / 2 - S > 0 ? KW - KW / 2 - S : 0;   // right neighbours needed
  constexpr int WIN = HL + SV + HR;
  constexpr int ROWS = S * RB + KH - S;          // input rows under a strip of RB output rows
  static_assert(HL <= SV && HR <= SV, "neighbours must come from the adjacent lane only");
  static_assert(KH >= S, "row window shorter than the row step");

  const int lane = threadIdx.x & 63;
  const int lpg = 1 << p.lpg_log2;
  const int lig = lane & (lpg - 1);
  const int grp = lane >> p.lpg_log2, gpw = 64 >> p.lpg_log2;   // group within the wave, groups per wave
  const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int x0 = lig * SV;                       // first input column this lane loads
  const int w0 = lig * V;                        // first output column this lane produces
  constexpr int HALO = KH - S;                   // input rows a strip shares with the strip above it

  // Request every input row of task `task` (one independent load per row: the wave pays the memory
  // latency once per strip).  Every load is issued unconditionally from an address clamped into the plane and
  // the value is replaced by zero afterwards where the row or column lies outside, so no branch (and no wait)
  // separates the loads.  Rows a strip shares with the strip above are not needed when that strip belongs to
  // the previous group of this wave (they are shuffled over afterwards): their loads are pointed at the first
  // row the lane does need, a line it fetches anyway.
  auto request = [&](int task, float (&v)[ROWS][SV]) {
    const bool task_ok = task < p.n_tasks;
    const int plane = task_ok ? task / p.strips : 0;
    const int strip = task_ok ? task - plane * p.strips : 0;
    const float* xp = X + (int64_t)plane * p.Hi * p.Wi;
    const int r0 = S * strip * RB - p.ph;
    const bool col_ok = task_ok && x0 < p.Wi;
    const bool from_prev = grp > 0 && strip > 0;
    const int xc = x0 < p.Wi ? x0 : 0;
#pragma unroll
    for (int a = 0; a < ROWS; ++a) {
      const int r = (a < HALO && from_prev) ? r0 + HALO : r0 + a;
      const float* row = xp + (int64_t)min(max(r, 0), p.Hi - 1) * p.Wi;
      if constexpr (VEC && SV == 4) {
        const float4 t = *reinterpret_cast<const float4*>(row + xc);
        v[a][0] = t.x; v[a][1] = t.y; v[a][2] = t.z; v[a][3] = t.w;
      } else {
#pragma unroll
        for (int e = 0; e < SV; ++e) v[a][e] = row[min(x0 + e, p.Wi - 1)];
      }
    }
#pragma unroll
    for (int a = 0; a < ROWS; ++a)
#pragma unroll
      for (int e = 0; e < SV; ++e) pin(v[a][e]);
#pragma unroll
    for (int a = 0; a < ROWS; ++a) {
      const int r = r0 + a;
      const bool row_ok = col_ok && r >= 0 && r < p.Hi && !(a < HALO && from_prev);
#pragma unroll
      for (int e = 0; e < SV; ++e)
        if (!(row_ok && (VEC || x0 + e < p.Wi))) v[a][e] = 0.f;
    }
  };
  auto finish = [&](int task, float (&v)[ROWS][SV], float (&wk)[KH][KW]) {
    const bool task_ok = task < p.n_tasks;
    const int plane = task_ok ? task / p.strips : 0;
    const int strip = task_ok ? task - plane * p.strips : 0;
    const int h0 = strip * RB;
    float* op = out + (int64_t)plane * p.Ho * p.Wo;
    const bool from_prev = grp > 0 && strip > 0;
    // shared rows come from the group above (every lane takes part in the shuffles)
#pragma unroll
    for (int a = 0; a < HALO; ++a)
#pragma unroll
      for (int e = 0; e < SV; ++e) {
        const float t = __shfl_up(v[ROWS - HALO + a][e], lpg, 64);
        if (from_prev) v[a][e] = t;
      }
    // the window's horizontal neighbours come from the adjacent lanes
    float left[ROWS][HL > 0 ? HL : 1], right[ROWS][HR > 0 ? HR : 1];
#pragma unroll
    for (int a = 0; a < ROWS; ++a) {
#pragma unroll
      for (int j = 0; j < HL; ++j) {
        const float t = __shfl_up(v[a][SV - HL + j], 1, 64);
        left[a][j] = lig == 0 ? 0.f : t;
      }
#pragma unroll
      for (int j = 0; j < HR; ++j) {
        const float t = __shfl_down(v[a][j], 1, 64);
        right[a][j] = lig == lpg - 1 ? 0.f : t;
      }
    }
    auto win = [&](int a, int i) -> float {      // column i of the widened row a (compile-time indices after unrolling)
      return i < HL ? left[a][i] : (i < HL + SV ? v[a][i - HL] : right[a][i - HL - SV]);
    };
    if constexpr (MODE == 0) {
#pragma unroll
      for (int i = 0; i < RB; ++i) {
        const int h = h0 + i;
        float acc[V];
#pragma unroll
        for (int o = 0; o < V; ++o) {
          acc[o] = 0.f;
#pragma unroll
          for (int a = 0; a < KH; ++a)
#pragma unroll
            for (int b = 0; b < KW; ++b) acc[o] = fmaf(wk[a][b], win(S * i + a, S * o + b), acc[o]);
        }
        if (task_ok && h < p.Ho) {
          float* o = op + (int64_t)h * p.Wo + w0;
          if (V == 2 && (p.Wo & 1) == 0) {
            if (w0 < p.Wo) *reinterpret_cast<float2*>(o) = make_float2(acc[0], acc[1]);
          } else if (V == 4 && (p.Wo & 3) == 0) {
            if (w0 < p.Wo) *reinterpret_cast<float4*>(o) = make_float4(acc[0], acc[1], acc[2], acc[3]);
          } else {
#pragma unroll
            for (int e = 0; e < V; ++e)
              if (w0 + e < p.Wo) o[e] = acc[e];
          }
        }
      }
    } else {
      // sums of G * window over the strip, per tap; Wt is G here, laid out like the forward result
      const float* gp = Wt + (int64_t)plane * p.Ho * p.Wo;
      float gv[RB][V];
      const bool pair = V == 2 && (p.Wo & 1) == 0;    // (clamped addresses, zeros selected afterwards: see request)
      const int wc = w0 < p.Wo ? w0 : 0;
#pragma unroll
      for (int i = 0; i < RB; ++i) {
        const float* grow = gp + (int64_t)min(h0 + i, p.Ho - 1) * p.Wo;
        if (pair) {
          const float2 t = *reinterpret_cast<const float2*>(grow + wc);
          gv[i][0] = t.x; gv[i][V - 1] = t.y;
        } else {
#pragma unroll
          for (int o = 0; o < V; ++o) gv[i][o] = grow[min(w0 + o, p.Wo - 1)];
        }
      }
#pragma unroll
      for (int i = 0; i < RB; ++i)
#pragma unroll
        for (int o = 0; o < V; ++o) pin(gv[i][o]);
#pragma unroll
      for (int i = 0; i < RB; ++i)
#pragma unroll
        for (int o = 0; o < V; ++o)
          if (!(task_ok && h0 + i < p.Ho && w0 + o < p.Wo)) gv[i][o] = 0.f;
#pragma unroll
      for (int i = 0; i < RB; ++i)
#pragma unroll
        for (int o = 0; o < V; ++o)
#pragma unroll
          for (int a = 0; a < KH; ++a)
#pragma unroll
            for (int b = 0; b < KW; ++b) wk[a][b] = fmaf(gv[i][o], win(S * i + a, S * o + b), wk[a][b]);
      // add up the lanes of the group (a fixed tree, so the result does not depend on scheduling)
#pragma unroll
      for (int a = 0; a < KH; ++a)
#pragma unroll
        for (int b = 0; b < KW; ++b) {
          float v = wk[a][b];
          for (int d = 1; d < lpg; d <<= 1) v += __shfl_xor(v, d, 64);
          if (lig == 0 && task_ok) out[(int64_t)task * (KH * KW) + a * KW + b] = v;
        }
    }
  };

  // one strip per group; every lane of the wave runs both phases so that the shuffles stay uniform
  float v[ROWS][SV];
  const int task = wave * gpw + grp;
  // the window's weights are requested ahead of the rows, so that they arrive within the same round trip
  float wk[KH][KW];
  const int c = (task < p.n_tasks ? task / p.strips : 0) % p.C;
#pragma unroll
  for (int a = 0; a < KH; ++a)
#pragma unroll
    for (int b = 0; b < KW; ++b) wk[a][b] = MODE == 0 ? Wt[c * p.ws_c + a * p.ws_kh + b * p.ws_kw] : 0.f;
  request(task, v);
  finish(task, v, wk);
  (void)WIN;
}

// Backward-data of the 3x3 stride-2 (pad 1) per-channel window: dX[y][x] = sum over the (h,w,kh,kw) with
// 2h+kh-1 = y, 2w+kw-1 = x of G[h][w] * W[kh][kw]: one term when y and x are even, two when one is odd, four
// when both are.  A group of lanes owns RB rows of G of one plane (plus the row below them) and writes the
// 2*RB rows of dX above them; a lane loads 2 columns of G per row, takes the third from its right neighbour
// with a shuffle and writes 4 columns of dX per row.  G is read once (plus one halo row per strip), dX written once.
template <int RB>
__global__ __launch_bounds__(256) void depthwise_s2k3_bwd_data(const DwParams p, const float* __restrict__ G,
                                                               const float* __restrict__ Wt, float* __restrict__ dX) {
  const int lane = threadIdx.x & 63;
  const int lpg = 1 << p.lpg_log2;
  const int lig = lane & (lpg - 1);
  const int grp = lane >> p.lpg_log2, gpw = 64 >> p.lpg_log2;
  const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int task = wave * gpw + grp;
  const bool task_ok = task < p.n_tasks;
  const int plane = task_ok ? task / p.strips : 0;
  const int strip = task_ok ? task - plane * p.strips : 0;
  const int h0 = strip * RB, c = plane % p.C;
  const int w0 = 2 * lig;                          // first of the lane's two columns of G
  const float* gp = G + (int64_t)plane * p.Ho * p.Wo;
  float w[3][3];                                   // requested ahead of G: one round trip for both
#pragma unroll
  for (int a = 0; a < 3; ++a)
#pragma unroll
    for (int b = 0; b < 3; ++b) w[a][b] = Wt[c * p.ws_c + a * p.ws_kh + b * p.ws_kw];
  float g[RB + 1][2], gn[RB + 1];
  const int wc = w0 < p.Wo ? w0 : 0;               // (Wo is even here) clamped addresses, zeros selected afterwards
#pragma unroll
  for (int r = 0; r <= RB; ++r) {
    const float2 t = *reinterpret_cast<const float2*>(gp + (int64_t)min(h0 + r, p.Ho - 1) * p.Wo + wc);
    g[r][0] = t.x; g[r][1] = t.y;
  }
#pragma unroll
  for (int r = 0; r <= RB; ++r) { pin(g[r][0]); pin(g[r][1]); }
#pragma unroll
  for (int r = 0; r <= RB; ++r)
    if (!(task_ok && h0 + r < p.Ho && w0 < p.Wo)) g[r][0] = g[r][1] = 0.f;
#pragma unroll
  for (int r = 0; r <= RB; ++r) {
    const float t = __shfl_down(g[r][0], 1, 64);
    gn[r] = (lig == lpg - 1 || w0 + 2 >= p.Wo) ? 0.f : t;
  }
  float* xp = dX + (int64_t)plane * p.Hi * p.Wi;
#pragma unroll
  for (int r = 0; r < RB; ++r) {
    const int h = h0 + r;
    if (!task_ok || h >= p.Ho || 4 * lig >= p.Wi) continue;
    const float a0 = g[r][0], a1 = g[r][1], a2 = gn[r];                  // G row h, columns w0, w0+1, w0+2
    const float b0 = g[r + 1][0], b1 = g[r + 1][1], b2 = gn[r + 1];      // G row h+1
    // dX row 2h: only kh = 1 reaches it
    const float4 even = make_float4(a0 * w[1][1], fmaf(a1, w[1][0], a0 * w[1][2]), a1 * w[1][1], fmaf(a2, w[1][0], a1 * w[1][2]));
    // dX row 2h+1: kh = 2 from G row h, kh = 0 from G row h+1
    const float4 odd = make_float4(
        fmaf(b0, w[0][1], a0 * w[2][1]),
        fmaf(b1, w[0][0], fmaf(b0, w[0][2], fmaf(a1, w[2][0], a0 * w[2][2]))),
        fmaf(b1, w[0][1], a1 * w[2][1]),
        fmaf(b2, w[0][0], fmaf(b1, w[0][2], fmaf(a2, w[2][0], a1 * w[2][2]))));
    *reinterpret_cast<float4*>(xp + (int64_t)(2 * h) * p.Wi + 4 * lig) = even;
    *reinterpret_cast<float4*>(xp + (int64_t)(2 * h + 1) * p.Wi + 4 * lig) = odd;
  }
}

// Backward-weight, second stage: dW[c][tap] = sum over the images and strips of the partial sums.  One block per
// channel; thread j adds the partials j, j+256, ... of the channel, then the threads' sums are added in a
// fixed tree, so the result does not depend on scheduling.
__global__ __launch_bounds__(256) void depthwise_bwd_weight_reduce(const DwParams p, const float* __restrict__ partial,
                                                                   float* __restrict__ dW, int KW) {
  constexpr int T = 9;
  __shared__ float sums[T][256];
  const int c = blockIdx.x, tid = threadIdx.x;
  const int per_c = (p.planes / p.C) * p.strips;      // partials of one channel
  float s[T];
#pragma unroll
  for (int t = 0; t < T; ++t) s[t] = 0.f;
  for (int q = tid; q < per_c; q += 256) {
    const int n = q / p.strips, st = q - n * p.strips;
    const float* src = partial + ((int64_t)(n * p.C + c) * p.strips + st) * T;
#pragma unroll
    for (int t = 0; t < T; ++t) s[t] += src[t];
  }
#pragma unroll
  for (int t = 0; t < T; ++t) sums[t][tid] = s[t];
  __syncthreads();
  for (int half = 128; half > 0; half >>= 1) {
    if (tid < half)
#pragma unroll
      for (int t = 0; t < T; ++t) sums[t][tid] += sums[t][tid + half];
    __syncthreads();
  }
  if (tid < T) dW[c * p.ws_c + (tid / KW) * p.ws_kh + (tid % KW) * p.ws_kw] = sums[tid][0];
}

constexpr int kStripRows = 7;   // output rows per strip: 15 input rows of a 3x3 stride-2 window in registers

template <int KH, int KW, int S, int V, int MODE>
void launch_dw(const DwParams& p, const float* X, const float* W, float* out, hipStream_t s) {
  const int groups_per_wave = 64 >> p.lpg_log2;
  const int waves = (p.n_tasks + groups_per_wave - 1) / groups_per_wave;
  const int wpb = 4;
  const int blocks = (waves + wpb - 1) / wpb;
  if (p.vec_ok)
    hipLaunchKernelGGL((depthwise_stream<KH, KW, S, V, kStripRows, MODE, true>), dim3(blocks), dim3(64 * wpb), 0, s, p, X, W, out);
  else
    hipLaunchKernelGGL((depthwise_stream<KH, KW, S, V, kStripRows, MODE, false>), dim3(blocks), dim3(64 * wpb), 0, s, p, X, W, out);
}

}  // namespace

// Can the stream kernels take this pass?  (fp32, one channel per group, no cyclic axes, pads equal to K/2, a
// window/stride pair that is instantiated, rows no wider than a wave.)  Forward: 3x3 at stride 1 or 2.
// Backward-data and backward-weight: 3x3 at stride 2 with an input exactly twice the output.
bool bandwidth_supports(const syno_plan* p, int which) {
  if (!p->conv_like) return false;
  if (p->in_dtype != SYNO_F32 || p->out_dtype != SYNO_F32) return false;
  const ConvLike& c = p->conv;
  if (c.Og != 1 || c.Cg != 1 || c.h_wrap || c.w_wrap) return false;
  if (c.sh != c.sw || c.ph != c.KH / 2 || c.pw != c.KW / 2) return false;
  const bool inst = (c.KH == 3 && c.KW == 3 && (c.sh == 1 || c.sh == 2));
  if (!inst) return false;
  const int V = c.sh == 2 ? 2 : 4;
  if ((c.Wo + V - 1) / V > 64) return false;
  if (which == SYNO_FWD) return true;
  if (c.sh != 2 || c.Hi != 2 * c.Ho || c.Wi != 2 * c.Wo || (c.Wo & 1)) return false;
  return c.ws_g >= 0 && c.ws_kh >= 0 && c.ws_kw >= 0;
}

// Fills the launch record: the kernel parameters, and for backward-weight the workspace that keeps one partial
// sum per strip and tap.
void bandwidth_configure(syno_plan* plan, int which) {
  const ConvLike& c = plan->conv;
  const int V = c.sh == 2 ? 2 : 4;
  DwParams p{};
  p.planes = c.N * c.G; p.C = c.G;
  p.Hi = c.Hi; p.Wi = c.Wi; p.Ho = c.Ho; p.Wo = c.Wo; p.ph = c.ph; p.pw = c.pw;
  const int lanes = (c.Wo + V - 1) / V;
  p.lpg_log2 = 0;
  while ((1 << p.lpg_log2) < lanes) ++p.lpg_log2;
  p.rb = kStripRows;
  p.strips = (c.Ho + p.rb - 1) / p.rb;
  p.n_tasks = p.planes * p.strips;
  p.ws_c = c.ws_g; p.ws_kh = c.ws_kh; p.ws_kw = c.ws_kw;
  p.vec_ok = (c.Wi % (c.sw * V) == 0) && ((c.Hi * c.Wi) % 4 == 0) && (c.Wi % 4 == 0);
  Launch& L = plan->launch[which];
  static_assert(sizeof(DwParams) <= sizeof(L.params), "parameter record does not fit");
  memcpy(L.params, &p, sizeof p);
  L.params_ready = true;
  L.workspace = which == SYNO_BWD_WEIGHT ? (size_t)c.N * c.G * p.strips * c.KH * c.KW * sizeof(float) : 0;
}

syno_status launch_bandwidth(const syno_plan* plan, int which, const void* A, const void* B, void* out, void* ws,
                             hipStream_t stream) {
  if (!plan->launch[which].params_ready) return SYNO_ERR_UNSUPPORTED;
  const ConvLike& c = plan->conv;
  DwParams p;
  memcpy(&p, plan->launch[which].params, sizeof p);
  if (which == SYNO_FWD) {
    const float* X = static_cast<const float*>(A);
    const float* W = static_cast<const float*>(B);
    float* O = static_cast<float*>(out);
    if (c.sh == 2) launch_dw<3, 3, 2, 2, 0>(p, X, W, O, stream);
    else launch_dw<3, 3, 1, 4, 0>(p, X, W, O, stream);
  } else if (which == SYNO_BWD_DATA) {
    // A = G, B = W, out = dX
    const int groups_per_wave = 64 >> p.lpg_log2;
    const int waves = (p.n_tasks + groups_per_wave - 1) / groups_per_wave;
    hipLaunchKernelGGL((depthwise_s2k3_bwd_data<kStripRows>), dim3((waves + 3) / 4), dim3(256), 0, stream, p,
                       static_cast<const float*>(A), static_cast<const float*>(B), static_cast<float*>(out));
  } else {
    // A = G, B = X (the lowered forms take the upstream gradient first), out = dW, ws = partial sums
    if (!ws) return SYNO_ERR_WORKSPACE;
    launch_dw<3, 3, 2, 2, 2>(p, static_cast<const float*>(B), static_cast<const float*>(A), static_cast<float*>(ws), stream);
    hipLaunchKernelGGL(depthwise_bwd_weight_reduce, dim3(p.C), dim3(256), 0, stream, p, static_cast<const float*>(ws),
                       static_cast<float*>(out), 3);
  }
  return hipGetLastError() == hipSuccess ? SYNO_OK : SYNO_ERR_HIP;
}

}  // namespace syno
