// Bandwidth-bound family, second member: a window whose iterator is Shared with the weight but not
// Reduced, so that it survives as an output axis (the first stage of Operator 1, Fig. 7 of the paper):
//
//   Z[n,d,g,k,h,w] = sum_c X[n, g*Cg+c, h, w+k-pw] * Wt[d,g,c,k]        (zero outside the row), pw = K/2
//
// and its two gradients
//
//   dX[n, g*Cg+c, h, x] = sum_{d,k} G[n,d,g,k,h, x-k+pw] * Wt[d,g,c,k]
//   dW[d,g,c,k]         = sum_{n,h,w} G[n,d,g,k,h,w] * X[n, g*Cg+c, h, w+k-pw].
//
// Each output of Z costs Cg multiply-adds and the result is K*D*G/(G*Cg) times the size of X, so at the
// layer shapes of interest the pass is a stream: read X once, write Z once.  Lanes own runs of V adjacent
// pixels of one row (one vector load / store per plane); the K-1 window neighbours at the ends of a run are
// single loads that hit the lines the adjacent lanes fetch; the few weights a workgroup needs sit in LDS
// and are read as broadcasts; accumulation is fp32 in registers.
#include <hip/hip_runtime.h>

#include <cstring>

#include <algorithm>

#include "plan.h"

namespace syno {
namespace {

struct SwParams {
  int32_t N, D, G, K, H, W, Cg;
  int32_t ws_d, ws_g, ws_c, ws_k;
  int32_t HW, runs_per_plane, n_runs;   // a run = V adjacent pixels of one row; n_runs = N * HW / V
  int32_t chunks, runs_per_chunk;       // backward-weight: runs are dealt to `chunks` workgroups per (g, tile)
  int32_t w_elems;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// fp32 -> bf16, round to nearest even: the conversion the hardware provides (v_cvt_pk_bf16_f32), two at a time.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <bool BF>
__device__ __forceinline__ float load_one(const void* base, int64_t off) {
  if constexpr (BF) return bf16_to_f32(static_cast<const uint16_t*>(base)[off]);
  else return static_cast<const float*>(base)[off];
}

// V adjacent elements starting at `off` (a multiple of V) as one vector access.
template <int V, bool BF>
__device__ __forceinline__ void load_run(const void* base, int64_t off, float* v) {
  if constexpr (BF) {
    const uint16_t* p = static_cast<const uint16_t*>(base) + off;
    if constexpr (V == 4) {
      const uint2 t = *reinterpret_cast<const uint2*>(p);
      v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
      v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
    } else if constexpr (V == 2) {
      const uint32_t t = *reinterpret_cast<const uint32_t*>(p);
      v[0] = __uint_as_float(t << 16); v[1] = __uint_as_float(t & 0xffff0000u);
    } else {
      v[0] = bf16_to_f32(*p);
    }
  } else {
    const float* p = static_cast<const float*>(base) + off;
    if constexpr (V == 4) {
      const float4 t = *reinterpret_cast<const float4*>(p);
      v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else if constexpr (V == 2) {
      const float2 t = *reinterpret_cast<const float2*>(p);
      v[0] = t.x; v[1] = t.y;
    } else {
      v[0] = *p;
    }
  }
}

template <int V, bool BF>
__device__ __forceinline__ void store_run(void* base, int64_t off, const float* v) {
  if constexpr (BF) {
    uint16_t* p = static_cast<uint16_t*>(base) + off;
    if constexpr (V == 4) {
      uint2 t;
      t.x = pack_bf16x2(v[0], v[1]);
      t.y = pack_bf16x2(v[2], v[3]);
      *reinterpret_cast<uint2*>(p) = t;
    } else if constexpr (V == 2) {
      *reinterpret_cast<uint32_t*>(p) = pack_bf16x2(v[0], v[1]);
    } else {
      *p = (uint16_t)pack_bf16x2(v[0], 0.f);
    }
  } else {
    float* p = static_cast<float*>(base) + off;
    if constexpr (V == 4) *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    else if constexpr (V == 2) *reinterpret_cast<float2*>(p) = make_float2(v[0], v[1]);
    else *p = v[0];
  }
}

// The K+V-1 elements of row `row_off` (offset of the row's first element) that the windows of the run
// starting at column w0 touch: columns w0-PW .. w0+V+K-2-PW, zero outside [0, W).  Branch-free: a neighbour
// outside the row is loaded from the nearest column inside it and replaced by zero afterwards, so that all
// loads of a lane can be in flight together.
template <int K, int V, bool BF>
__device__ __forceinline__ void load_window(const void* base, int64_t row_off, int w0, int W, float* win) {
  constexpr int PW = K / 2;
  load_run<V, BF>(base, row_off + w0, win + PW);
#pragma unroll
  for (int j = 0; j < PW; ++j) {
    const int x = w0 - PW + j;
    const float t = load_one<BF>(base, row_off + max(x, 0));
    win[j] = x >= 0 ? t : 0.f;
  }
#pragma unroll
  for (int j = 0; j < K - 1 - PW; ++j) {
    const int x = w0 + V + j;
    const float t = load_one<BF>(base, row_off + min(x, W - 1));
    win[PW + V + j] = x < W ? t : 0.f;
  }
}

// Keeps the compiler from sinking a load below this point: everything requested so far is in flight together.
template <int N>
__device__ __forceinline__ void pin(float (&v)[N]) {
#pragma unroll
  for (int i = 0; i < N; ++i) asm volatile("" : "+v"(v[i]));
}

constexpr int kThreads = 256;
constexpr int kDT = 8;    // forward: output-channel digits d a lane accumulates at once
constexpr int kCB = 8;    //          input channels whose windows are in flight together
constexpr int kCT = 16;   // backward-data: input channels c a lane accumulates at once
constexpr int kDB = 4;    //                d digits whose gradient runs are in flight together
constexpr int kWD = 4;    // backward-weight: d digits per lane ...
constexpr int kWC = 8;    // ... times input channels per lane

// ------------------------------------------------------------------------------------------------
// forward.  grid = (run blocks, G, d tiles)
// ------------------------------------------------------------------------------------------------
template <int K, int V, bool IBF, bool OBF>
__global__ __launch_bounds__(kThreads) void share_window_fwd(const SwParams p, const void* __restrict__ X,
                                                            const void* __restrict__ Wt, void* __restrict__ Z) {
  extern __shared__ float wl[];   // [Cg][kDT][K]
  const int g = blockIdx.y, d0 = blockIdx.z * kDT;
  for (int i = threadIdx.x; i < p.Cg * kDT * K; i += kThreads) {
    const int c = i / (kDT * K), r = i - c * (kDT * K), dt = r / K, k = r - dt * K;
    const int d = d0 + dt;
    wl[i] = d < p.D ? load_one<IBF>(Wt, (int64_t)d * p.ws_d + (int64_t)g * p.ws_g + (int64_t)c * p.ws_c +
                                            (int64_t)k * p.ws_k)
                    : 0.f;
  }
  __syncthreads();
  const int q = blockIdx.x * kThreads + threadIdx.x;
  if (q >= p.n_runs) return;
  const int n = q / p.runs_per_plane;
  const int pix0 = (q - n * p.runs_per_plane) * V;
  const int h = pix0 / p.W, w0 = pix0 - h * p.W;
  float acc[kDT][K][V];
#pragma unroll
  for (int a = 0; a < kDT; ++a)
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
      for (int v = 0; v < V; ++v) acc[a][k][v] = 0.f;
  const int64_t row0 = ((int64_t)n * p.G * p.Cg + (int64_t)g * p.Cg) * p.HW + (int64_t)h * p.W;
  for (int cb = 0; cb < p.Cg; cb += kCB) {
    // the windows of kCB channels are requested together: one memory round trip per batch
    float win[kCB][V + K - 1];
#pragma unroll
    for (int j = 0; j < kCB; ++j)
      load_window<K, V, IBF>(X, row0 + (int64_t)min(cb + j, p.Cg - 1) * p.HW, w0, p.W, win[j]);
#pragma unroll
    for (int j = 0; j < kCB; ++j) pin(win[j]);
#pragma unroll
    for (int j = 0; j < kCB; ++j) {
      if (cb + j < p.Cg) {
        const float* wc = wl + (cb + j) * (kDT * K);
#pragma unroll
        for (int a = 0; a < kDT; ++a)
#pragma unroll
          for (int k = 0; k < K; ++k) {
            const float wv = wc[a * K + k];
#pragma unroll
            for (int v = 0; v < V; ++v) acc[a][k][v] = fmaf(win[j][v + k], wv, acc[a][k][v]);
          }
      }
    }
  }
#pragma unroll
  for (int a = 0; a < kDT; ++a) {
    const int d = d0 + a;
    if (d < p.D) {
#pragma unroll
      for (int k = 0; k < K; ++k)
        store_run<V, OBF>(Z, ((((int64_t)n * p.D + d) * p.G + g) * K + k) * p.HW + pix0, acc[a][k]);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// backward-data.  grid = (run blocks, G, c tiles)
// ------------------------------------------------------------------------------------------------
template <int K, int V, bool IBF, bool OBF>
__global__ __launch_bounds__(kThreads) void share_window_bwd_data(const SwParams p, const void* __restrict__ Gr,
                                                                 const void* __restrict__ Wt,
                                                                 void* __restrict__ dX) {
  constexpr int PW = K / 2;
  extern __shared__ float wl[];   // [D][K][kCT]
  const int g = blockIdx.y, c0 = blockIdx.z * kCT;
  for (int i = threadIdx.x; i < p.D * K * kCT; i += kThreads) {
    const int d = i / (K * kCT), r = i - d * (K * kCT), k = r / kCT, ct = r - k * kCT;
    const int c = c0 + ct;
    wl[i] = c < p.Cg ? load_one<IBF>(Wt, (int64_t)d * p.ws_d + (int64_t)g * p.ws_g + (int64_t)c * p.ws_c +
                                             (int64_t)k * p.ws_k)
                     : 0.f;
  }
  __syncthreads();
  const int q = blockIdx.x * kThreads + threadIdx.x;
  if (q >= p.n_runs) return;
  const int n = q / p.runs_per_plane;
  const int pix0 = (q - n * p.runs_per_plane) * V;
  const int h = pix0 / p.W, w0 = pix0 - h * p.W;
  float acc[kCT][V];
#pragma unroll
  for (int a = 0; a < kCT; ++a)
#pragma unroll
    for (int v = 0; v < V; ++v) acc[a][v] = 0.f;
  for (int db = 0; db < p.D; db += kDB) {
    // dX at column x takes G of plane (d,g,k) at column x - k + PW: the run itself plus |PW - k| elements
    // beyond one of its ends.  The runs of kDB digits are requested together.
    float cen[kDB][K][V], edge[kDB][K][PW > 0 ? PW : 1];
#pragma unroll
    for (int j = 0; j < kDB; ++j) {
      const int d = min(db + j, p.D - 1);
#pragma unroll
      for (int k = 0; k < K; ++k) {
        const int shift = PW - k;
        const int64_t row = ((((int64_t)n * p.D + d) * p.G + g) * K + k) * p.HW + (int64_t)h * p.W;
        load_run<V, IBF>(Gr, row + w0, cen[j][k]);
#pragma unroll
        for (int t = 0; t < (shift > 0 ? shift : -shift); ++t) {
          const int x = shift > 0 ? w0 + V + t : w0 - 1 - t;
          const float e = load_one<IBF>(Gr, row + min(max(x, 0), p.W - 1));
          edge[j][k][t] = (x >= 0 && x < p.W) ? e : 0.f;
        }
      }
    }
#pragma unroll
    for (int j = 0; j < kDB; ++j)
#pragma unroll
      for (int k = 0; k < K; ++k) {
        pin(cen[j][k]);
        if (k != PW) pin(edge[j][k]);
      }
#pragma unroll
    for (int j = 0; j < kDB; ++j) {
      if (db + j < p.D) {
#pragma unroll
        for (int k = 0; k < K; ++k) {
          const int shift = PW - k;
          float gv[V];
#pragma unroll
          for (int v = 0; v < V; ++v) {
            const int t = v + shift;
            gv[v] = (t >= 0 && t < V) ? cen[j][k][t] : (t >= V ? edge[j][k][t - V] : edge[j][k][-t - 1]);
          }
          const float* wk = wl + ((db + j) * K + k) * kCT;
#pragma unroll
          for (int a = 0; a < kCT; ++a) {
            const float wv = wk[a];
#pragma unroll
            for (int v = 0; v < V; ++v) acc[a][v] = fmaf(gv[v], wv, acc[a][v]);
          }
        }
      }
    }
  }
#pragma unroll
  for (int a = 0; a < kCT; ++a) {
    const int c = c0 + a;
    if (c < p.Cg)
      store_run<V, OBF>(dX, ((int64_t)n * p.G * p.Cg + (int64_t)g * p.Cg + c) * p.HW + pix0, acc[a]);
  }
}

// ------------------------------------------------------------------------------------------------
// backward-weight.  One workgroup per (chunk of runs, g, tile of kWD x kWC weights); it leaves the sums over its
// runs in partial[chunk][weight offset], and a second kernel adds the chunks in a fixed order.  The tiles of one
// (chunk, g) read the same gradient planes and input rows; the grid is one-dimensional and decoded so that they
// are consecutive workgroups of the same XCD (workgroups go round-robin over the 8 XCDs), which makes the
// re-reads hit that XCD's L2 while it still holds the lines.
// ------------------------------------------------------------------------------------------------
template <int K, int V, bool IBF>
__global__ __launch_bounds__(kThreads) void share_window_bwd_weight(const SwParams p, const void* __restrict__ Gr,
                                                                   const void* __restrict__ X,
                                                                   float* __restrict__ partial) {
  constexpr int NACC = kWD * kWC * K;
  __shared__ float red[kThreads / 64][NACC];
  const int c_tiles = (p.Cg + kWC - 1) / kWC;
  const int tiles = c_tiles * ((p.D + kWD - 1) / kWD);
  int slot = blockIdx.x >> 3;
  const int tile = slot % tiles;
  slot /= tiles;
  const int g = slot % p.G;
  const int chunk = (slot / p.G) * 8 + (blockIdx.x & 7);
  if (chunk >= p.chunks) return;
  const int d0 = (tile / c_tiles) * kWD, c0 = (tile % c_tiles) * kWC;
  float acc[kWD][kWC][K];
#pragma unroll
  for (int a = 0; a < kWD; ++a)
#pragma unroll
    for (int b = 0; b < kWC; ++b)
#pragma unroll
      for (int k = 0; k < K; ++k) acc[a][b][k] = 0.f;
  const int q_end = min((chunk + 1) * p.runs_per_chunk, p.n_runs);
  for (int q = chunk * p.runs_per_chunk + threadIdx.x; q < q_end; q += kThreads) {
    const int n = q / p.runs_per_plane;
    const int pix0 = (q - n * p.runs_per_plane) * V;
    const int h = pix0 / p.W, w0 = pix0 - h * p.W;
    float xw[kWC][V + K - 1];
#pragma unroll
    for (int b = 0; b < kWC; ++b) {
      const int c = min(c0 + b, p.Cg - 1);   // channels past the end re-read the last one; their sums are dropped
      load_window<K, V, IBF>(X, ((int64_t)n * p.G * p.Cg + (int64_t)g * p.Cg + c) * p.HW + (int64_t)h * p.W, w0,
                             p.W, xw[b]);
    }
    // every gradient run of the tile is requested before the first one is used: one memory round trip
    float gv[kWD][K][V];
#pragma unroll
    for (int a = 0; a < kWD; ++a) {
      const int d = min(d0 + a, p.D - 1);   // digits past the end re-read the last plane; their sums are dropped
#pragma unroll
      for (int k = 0; k < K; ++k)
        load_run<V, IBF>(Gr, ((((int64_t)n * p.D + d) * p.G + g) * K + k) * p.HW + pix0, gv[a][k]);
    }
#pragma unroll
    for (int a = 0; a < kWD; ++a)
#pragma unroll
      for (int k = 0; k < K; ++k) pin(gv[a][k]);
#pragma unroll
    for (int a = 0; a < kWD; ++a)
#pragma unroll
      for (int k = 0; k < K; ++k)
#pragma unroll
        for (int b = 0; b < kWC; ++b)
#pragma unroll
          for (int v = 0; v < V; ++v) acc[a][b][k] = fmaf(gv[a][k][v], xw[b][v + k], acc[a][b][k]);
  }
  // Sum over the lanes of each wave by halving: at the step with lane mask m a lane passes one half of its
  // sums to lane^m and adds the half it receives, so the count of sums per lane halves while the count of lanes
  // added doubles; after masks 1..16 a lane holds NACC/32 complete half-wave sums, the last step adds the other
  // half-wave.  NACC/32 + ... + NACC/2 exchanges instead of 6 * NACC.
  static_assert(NACC % 32 == 0, "the sums must halve five times");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* v = &acc[0][0][0];
  int base = 0;
#pragma unroll
  for (int step = 0; step < 5; ++step) {
    const int half = NACC >> (step + 1);
    const bool upper = (lane >> step) & 1;
#pragma unroll
    for (int i = 0; i < half; ++i) {
      const float send = upper ? v[i] : v[i + half];
      const float keep = upper ? v[i + half] : v[i];
      v[i] = keep + __shfl_xor(send, 1 << step, 64);
    }
    base += upper ? half : 0;
  }
#pragma unroll
  for (int i = 0; i < NACC / 32; ++i) {
    v[i] += __shfl_xor(v[i], 32, 64);
    if (lane < 32) red[wave][base + i] = v[i];
  }
  __syncthreads();
  for (int i = threadIdx.x; i < NACC; i += kThreads) {
    const int a = i / (kWC * K), r = i - a * (kWC * K), b = r / K, k = r - b * K;
    const int d = d0 + a, c = c0 + b;
    if (d < p.D && c < p.Cg) {
      float s = red[0][i];
#pragma unroll
      for (int w = 1; w < kThreads / 64; ++w) s += red[w][i];
      partial[(int64_t)chunk * p.w_elems + (int64_t)d * p.ws_d + (int64_t)g * p.ws_g + (int64_t)c * p.ws_c +
              (int64_t)k * p.ws_k] = s;
    }
  }
}

// dW[e] = sum over the chunks of partial[chunk][e], in a fixed order: 16 lanes share one element, each adds
// every 16th chunk, and one lane adds the 16 sums.
__global__ __launch_bounds__(kThreads) void share_window_reduce(const float* __restrict__ partial,
                                                               float* __restrict__ dW, int chunks, int w_elems) {
  __shared__ float part[16][17];
  const int col = threadIdx.x & 15, j = threadIdx.x >> 4;
  const int e = blockIdx.x * 16 + col;
  float s = 0.f;
  if (e < w_elems)
    for (int c = j; c < chunks; c += 16) s += partial[(int64_t)c * w_elems + e];
  part[j][col] = s;
  __syncthreads();
  if (j == 0 && e < w_elems) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += part[i][col];
    dW[e] = t;
  }
}

int run_width(const ShareWindow& s) {
  if (s.K == 5) return s.W % 4 == 0 ? 4 : 1;      // (the 5-wide window is instantiated for runs of 4 and of 1)
  return s.W % 4 == 0 ? 4 : s.W % 2 == 0 ? 2 : 1;
}

SwParams fill(const syno_plan* plan) {
  const ShareWindow& s = plan->window;
  SwParams p{};
  p.N = s.N; p.D = s.D; p.G = s.G; p.K = s.K; p.H = s.H; p.W = s.W; p.Cg = s.Cg;
  p.ws_d = s.ws_d; p.ws_g = s.ws_g; p.ws_c = s.ws_c; p.ws_k = s.ws_k;
  p.HW = s.H * s.W;
  const int V = run_width(s);
  p.runs_per_plane = p.HW / V;
  p.n_runs = s.N * p.runs_per_plane;
  // backward-weight: about four workgroups per compute unit in total
  const int tiles = ((s.D + kWD - 1) / kWD) * ((s.Cg + kWC - 1) / kWC);
  const int per_lane_once = (p.n_runs + kThreads - 1) / kThreads;
  p.chunks = std::max(1, std::min(per_lane_once, 1024 / std::max(1, s.G * tiles)));
  p.runs_per_chunk = (p.n_runs + p.chunks - 1) / p.chunks;
  p.w_elems = (int32_t)plan->w_elems;
  return p;
}

template <int K, int V, bool IBF, bool OBF>
syno_status launch_typed(const SwParams& p, int which, const void* A, const void* B, void* out, void* ws,
                         hipStream_t stream) {
  const unsigned run_blocks = (unsigned)((p.n_runs + kThreads - 1) / kThreads);
  if (which == SYNO_FWD) {
    const dim3 grid(run_blocks, (unsigned)p.G, (unsigned)((p.D + kDT - 1) / kDT));
    hipLaunchKernelGGL((share_window_fwd<K, V, IBF, OBF>), grid, dim3(kThreads), sizeof(float) * p.Cg * kDT * K,
                       stream, p, A, B, out);
  } else if (which == SYNO_BWD_DATA) {
    const dim3 grid(run_blocks, (unsigned)p.G, (unsigned)((p.Cg + kCT - 1) / kCT));
    hipLaunchKernelGGL((share_window_bwd_data<K, V, IBF, OBF>), grid, dim3(kThreads),
                       sizeof(float) * p.D * K * kCT, stream, p, A, B, out);
  } else {
    const unsigned tiles = (unsigned)(((p.D + kWD - 1) / kWD) * ((p.Cg + kWC - 1) / kWC));
    const dim3 grid((unsigned)((p.chunks + 7) / 8 * 8) * (unsigned)p.G * tiles);
    hipLaunchKernelGGL((share_window_bwd_weight<K, V, IBF>), grid, dim3(kThreads), 0, stream, p, A, B,
                       static_cast<float*>(ws));
    hipLaunchKernelGGL(share_window_reduce, dim3((unsigned)((p.w_elems + 15) / 16)),
                       dim3(kThreads), 0, stream, static_cast<const float*>(ws), static_cast<float*>(out),
                       p.chunks, p.w_elems);
  }
  return hipGetLastError() == hipSuccess ? SYNO_OK : SYNO_ERR_HIP;
}

template <bool IBF, bool OBF>
syno_status launch_width(const SwParams& p, int V, int which, const void* A, const void* B, void* out, void* ws,
                         hipStream_t stream) {
  if (p.K == 5) {        // (the wider window keeps more sums per lane: runs of 4 and single elements only)
    if (V == 4) return launch_typed<5, 4, IBF, OBF>(p, which, A, B, out, ws, stream);
    return launch_typed<5, 1, IBF, OBF>(p, which, A, B, out, ws, stream);
  }
  switch (V) {
    case 4: return launch_typed<3, 4, IBF, OBF>(p, which, A, B, out, ws, stream);
    case 2: return launch_typed<3, 2, IBF, OBF>(p, which, A, B, out, ws, stream);
    default: return launch_typed<3, 1, IBF, OBF>(p, which, A, B, out, ws, stream);
  }
}

}  // namespace

bool window_supports(const syno_plan* plan, int which) {
  if (!plan->share_window) return false;
  const ShareWindow& s = plan->window;
  if (!((s.K == 3 || s.K == 5) && s.pw == s.K / 2)) return false;
  if (plan->in_dtype == SYNO_F32 && plan->out_dtype != SYNO_F32) return false;
  // the weights a workgroup keeps in LDS
  const size_t lds = sizeof(float) * (which == SYNO_FWD ? (size_t)s.Cg * kDT * s.K : (size_t)s.D * s.K * kCT);
  if (which != SYNO_BWD_WEIGHT && lds > 48 * 1024) return false;
  if (s.G > 65535 || (int64_t)((s.D + kWD - 1) / kWD) * ((s.Cg + kWC - 1) / kWC) * s.G > (1 << 20)) return false;
  return true;
}

void window_configure(syno_plan* plan, int which) {
  const SwParams p = fill(plan);
  Launch& L = plan->launch[which];
  static_assert(sizeof(SwParams) <= sizeof(L.params), "parameter record does not fit");
  memcpy(L.params, &p, sizeof p);
  L.params_ready = true;
  L.workspace = which == SYNO_BWD_WEIGHT ? sizeof(float) * (size_t)p.chunks * (size_t)p.w_elems : 0;
}

syno_status launch_window(const syno_plan* plan, int which, const void* A, const void* B, void* out, void* ws,
                          hipStream_t stream) {
  if (!plan->launch[which].params_ready) return SYNO_ERR_UNSUPPORTED;
  SwParams p;
  memcpy(&p, plan->launch[which].params, sizeof p);
  const int V = run_width(plan->window);
  const bool ibf = plan->in_dtype == SYNO_BF16;
  const bool obf = which != SYNO_BWD_WEIGHT && plan->out_dtype == SYNO_BF16;
  if (ibf && obf) return launch_width<true, true>(p, V, which, A, B, out, ws, stream);
  if (ibf) return launch_width<true, false>(p, V, which, A, B, out, ws, stream);
  return launch_width<false, false>(p, V, which, A, B, out, ws, stream);
}

}  // namespace syno
