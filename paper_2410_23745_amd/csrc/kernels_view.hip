// Bandwidth-bound family, third member: graphs without Unfold and with at most a few sum points per output -
// pure views (Shift, Split, Merge, Stride, Expand and Share in any combination) and small gather-and-add
// operators (block sums, pools) - forward pass,
//
//   out[o] = sum_r X[offX(o,r)] * W[offW(o,r)]
//
// for one-to-one views backward-data as the scatter dX[offX(o)] = G[o] * W[offW(o)], and the other gradients
// (backward-weight; backward-data of views that repeat or skip elements of X) as gathers: every target element is
// the sum, in a fixed order, of the products of the iterators that do not select it.
//
// When every tensor axis is an affine function of digits of the iterators - wrapped (Shift) only over digits of
// one iterator - both offsets are sums of one small table per iterator (plan.h, ViewStream); the tables of the
// Reduce iterators are folded into one table over the sum points.
// Every workgroup builds the tables in LDS from the record (a few hundred entries), then each lane takes a run
// of V adjacent elements of the innermost output axis: the outer axes are decoded once per run, the innermost
// axis is a table walk, the result leaves as one vector store.  The loads follow whatever order the view imposes.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <string>
#include <type_traits>
#include <vector>

#include "plan.h"

namespace syno {
namespace {

constexpr int kThreads = 256;

struct ViewParams {
  ViewStream vs;
  int32_t tab_off[2 * kMaxAxes]; // start of iterator i's table (entries, X table; the W table follows at +tab_total)
  uint32_t magic[kMaxAxes];      // division_magic(size[i]) of the output axes
  int32_t tab_total;             // entries of all iterator tables
  int32_t n_free, free_off;      // sum points per output; start of the folded table over them (X; W at +tab_total)
  int32_t scratch_off;           // start (entries, a multiple of 4) of the waves' exchange areas behind the two tables
  int64_t n_runs;                // out elements / V
  int32_t max_blocks;            // cap on the grid (the kernel walks the runs in a grid-stride loop)
};

__device__ __forceinline__ uint32_t div_magic(uint32_t n, uint32_t d, uint32_t magic) {
  return d < 2 ? n : __umulhi(n, magic) >> (31 - __clz((int)(d - 1)));
}

template <bool BF>
__device__ __forceinline__ float load_one(const void* base, int64_t off) {
  if constexpr (BF) return __uint_as_float((uint32_t)static_cast<const uint16_t*>(base)[off] << 16);
  else return static_cast<const float*>(base)[off];
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
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
    } else {
      *p = (uint16_t)pack_bf16x2(v[0], 0.f);
    }
  } else {
    float* p = static_cast<float*>(base) + off;
    if constexpr (V == 4) *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    else *p = v[0];
  }
}

// V adjacent elements starting at a multiple of V (one vector load when V = 4)
template <int V, bool BF>
__device__ __forceinline__ void load_run(const void* base, int64_t off, float* v) {
  if constexpr (V == 4 && BF) {
    const uint2 t = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(base) + off);
    v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
    v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
  } else if constexpr (V == 4) {
    const float4 t = *reinterpret_cast<const float4*>(static_cast<const float*>(base) + off);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  } else {
    v[0] = load_one<BF>(base, off);
  }
}

template <bool BF>
__device__ __forceinline__ void store_one(void* base, int64_t off, float v) {
  if constexpr (BF) static_cast<uint16_t*>(base)[off] = (uint16_t)pack_bf16x2(v, 0.f);
  else static_cast<float*>(base)[off] = v;
}

// Contribution of iterator `axis` at index o to the X offset (off[0]) and the W offset (off[1]).
__host__ __device__ inline void table_entry(const ViewStream& vs, int axis, int o, int (&off)[2]) {
  off[0] = off[1] = 0;
  for (int gi = 0; gi < vs.n_groups; ++gi) {
    const ViewGroup g = vs.group[gi];
    int partial = 0;
    const bool mine = g.axis == axis;          // the group's constant (and its wrap) are charged to one axis only
    for (int t = 0; t < vs.n_terms; ++t) {
      const ViewTerm tm = vs.term[t];
      if (tm.group == gi && tm.axis == axis) partial += tm.coef * ((o / tm.div) % tm.size);
    }
    if (g.wrap > 0) {
      if (mine) off[g.tensor] += ((partial + g.c) % g.wrap) * g.stride;
    } else {
      off[g.tensor] += (partial + (mine ? g.c : 0)) * g.stride;
    }
  }
}

// Every workgroup builds the tables in LDS: tab[tab_off[i] + o] (X) and tab[tab_total + tab_off[i] + o] (W) for every
// iterator i, then the folded table over the sum points at free_off.  Ends with a barrier.
__device__ __forceinline__ void build_tables(const ViewStream& vs, const int32_t* tab_off, int free_off, int n_free,
                                             int tab_total, int* tab) {
  const int n_iter = vs.n_axes + vs.n_red;
  for (int idx = threadIdx.x; idx < free_off; idx += kThreads) {
    int axis = 0;
    while (axis + 1 < n_iter && idx >= tab_off[axis + 1]) ++axis;
    int off[2];
    table_entry(vs, axis, idx - tab_off[axis], off);
    tab[idx] = off[0];
    tab[tab_total + idx] = off[1];
  }
  __syncthreads();
  // sum point q (Reduce iterators row-major, the order of the loop nest) -> the sum of its iterators' entries
  for (int q = threadIdx.x; q < n_free; q += kThreads) {
    int rest = q, fx = 0, fw = 0;
    for (int j = vs.n_red - 1; j >= 0; --j) {
      const int sz = vs.size[vs.n_axes + j], d = rest % sz;
      rest /= sz;
      fx += tab[tab_off[vs.n_axes + j] + d];
      fw += tab[tab_total + tab_off[vs.n_axes + j] + d];
    }
    tab[free_off + q] = fx;
    tab[tab_total + free_off + q] = fw;
  }
  __syncthreads();
}

// SCATTER: backward-data of a one-to-one view.  X is then the upstream gradient, shaped like the forward result and
// read in runs, and `out` is dX: dX[offX(o)] = G[o] * W[offW(o)], every element written exactly once.
template <int V, bool IBF, bool OBF, bool SCATTER>
__global__ __launch_bounds__(kThreads) void view_stream(const ViewParams p, const void* __restrict__ X,
                                                        const void* __restrict__ Wt, void* __restrict__ out) {
  extern __shared__ __align__(16) int tab[];   // [2][tab_total]: X offsets, then W offsets; then the waves' exchange areas
  const ViewStream& vs = p.vs;
  build_tables(vs, p.tab_off, p.free_off, p.n_free, p.tab_total, tab);
  const int last = vs.n_axes - 1;
  const uint32_t runs_per_row = (uint32_t)vs.size[last] / V;
  const int* const tx_last = tab + p.tab_off[last];
  if constexpr (V == 4) {
    if (p.n_free == 1) {
      // One product per element.  A lane decodes one run of 4 elements, but a wave touching memory run by run
      // would spread every load over 1 KB of the view's source.  So the wave exchanges what its lanes computed
      // through a 256-entry area in LDS and then works element by element: pass v takes the wave's elements
      // 64v .. 64v+63, adjacent lanes on adjacent elements, for the loads through the view (forward), the stores
      // through it (scatter) and the other side alike.  Every lane of the wave goes through every pass (the loop
      // is uniform per wave; lanes past the end decode the last run again and only their stores are masked).
      const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
      int* const ex = tab + p.scratch_off + wave * (3 * 256);     // X offsets | W offsets or values | (scatter) values
      int* const ew = ex + 256;
      const int64_t n_elems = p.n_runs * 4;
      // Several chunks of 64 runs per pass of the loop: the chunks' offsets go through the exchange area one after
      // the other (LDS is in order within a wave, so a chunk's writes follow the reads of the chunk before), then
      // all their elements' loads (or stores) are in flight together.  Measured: two chunks are best for the
      // gathering forward pass (a third and fourth cost registers and gain nothing), four for the scatter.
      constexpr int H = SCATTER ? 4 : 2;
      for (int64_t run0 = ((int64_t)blockIdx.x * kThreads + wave * 64) * H; run0 < p.n_runs;
           run0 += (int64_t)gridDim.x * kThreads * H) {
        int offx[H][4], offw[H][4];     // per element of pass (h, v): X offset; W offset (forward) or value bits (scatter)
#pragma unroll
        for (int h = 0; h < H; ++h) {
          const int64_t mine = run0 + 64 * h + lane;
          const int64_t run = mine < p.n_runs ? mine : p.n_runs - 1;
          uint32_t rest = (uint32_t)run;
          const uint32_t row = div_magic(rest, runs_per_row, p.magic[last]);
          const int w0 = (int)(rest - row * runs_per_row) * 4;
          rest = row;
          int bx = 0, bw = 0;
          for (int i = last - 1; i >= 0; --i) {
            const uint32_t sz = (uint32_t)vs.size[i];
            const uint32_t q = div_magic(rest, sz, p.magic[i]);
            const int o = (int)(rest - q * sz);
            rest = q;
            bx += tab[p.tab_off[i] + o];
            bw += tab[p.tab_total + p.tab_off[i] + o];
          }
          bx += tab[p.free_off];                      // the single sum point (Reduce iterators of size 1, if any)
          bw += tab[p.tab_total + p.free_off];
          const int* tx = tx_last + w0;
          const int* tw = tx + p.tab_total;
          *reinterpret_cast<int4*>(ex + 4 * lane) = make_int4(bx + tx[0], bx + tx[1], bx + tx[2], bx + tx[3]);
          if constexpr (SCATTER) {
            float g[4];
            load_run<4, IBF>(X, run * 4, g);
#pragma unroll
            for (int v = 0; v < 4; ++v) g[v] *= load_one<IBF>(Wt, bw + tw[v]);
            *reinterpret_cast<float4*>(ew + 4 * lane) = make_float4(g[0], g[1], g[2], g[3]);
          } else {
            *reinterpret_cast<int4*>(ew + 4 * lane) = make_int4(bw + tw[0], bw + tw[1], bw + tw[2], bw + tw[3]);
          }
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            offx[h][v] = ex[64 * v + lane];
            offw[h][v] = ew[64 * v + lane];
          }
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
        }
        const int64_t e0 = run0 * 4 + lane;
        if constexpr (SCATTER) {
#pragma unroll
          for (int h = 0; h < H; ++h)
#pragma unroll
            for (int v = 0; v < 4; ++v)
              if (e0 + 256 * h + 64 * v < n_elems) store_one<OBF>(out, offx[h][v], __int_as_float(offw[h][v]));
        } else {
          // every load is requested before the first value is used (the empty asm keeps the compiler from sinking
          // loads under the stores' bounds tests, where each would be waited for on its own)
          float val[H][4], wv[H][4];
#pragma unroll
          for (int h = 0; h < H; ++h)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              val[h][v] = load_one<IBF>(X, offx[h][v]);
              wv[h][v] = load_one<IBF>(Wt, offw[h][v]);
            }
#pragma unroll
          for (int h = 0; h < H; ++h)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              asm volatile("" : "+v"(val[h][v]), "+v"(wv[h][v]));
              val[h][v] *= wv[h][v];
            }
#pragma unroll
          for (int h = 0; h < H; ++h)
#pragma unroll
            for (int v = 0; v < 4; ++v)
              if (e0 + 256 * h + 64 * v < n_elems) store_one<OBF>(out, e0 + 256 * h + 64 * v, val[h][v]);
        }
      }
      return;
    }
  }
  for (int64_t run = (int64_t)blockIdx.x * kThreads + threadIdx.x; run < p.n_runs; run += (int64_t)gridDim.x * kThreads) {
    uint32_t rest = (uint32_t)run;
    const uint32_t row = div_magic(rest, runs_per_row, p.magic[last]);
    const int w0 = (int)(rest - row * runs_per_row) * V;
    rest = row;
    int bx = 0, bw = 0;
    for (int i = last - 1; i >= 0; --i) {
      const uint32_t s = (uint32_t)vs.size[i];
      const uint32_t q = div_magic(rest, s, p.magic[i]);
      const int o = (int)(rest - q * s);
      rest = q;
      bx += tab[p.tab_off[i] + o];
      bw += tab[p.tab_total + p.tab_off[i] + o];
    }
    float r[V];
    const int* tx = tx_last + w0;
    const int* tw = tx + p.tab_total;
    if constexpr (SCATTER) {
      load_run<V, IBF>(X, run * V, r);
#pragma unroll
      for (int v = 0; v < V; ++v) r[v] *= load_one<IBF>(Wt, bw + tw[v]);
#pragma unroll
      for (int v = 0; v < V; ++v) store_one<OBF>(out, bx + tx[v], r[v]);
      continue;
    }
    if (p.n_free == 1) {
      bx += tab[p.free_off];                        // the single sum point (Reduce iterators of size 1, if any)
      bw += tab[p.tab_total + p.free_off];
#pragma unroll
      for (int v = 0; v < V; ++v) r[v] = load_one<IBF>(X, bx + tx[v]) * load_one<IBF>(Wt, bw + tw[v]);
    } else {
      int ox[V], ow[V];
#pragma unroll
      for (int v = 0; v < V; ++v) { ox[v] = bx + tx[v]; ow[v] = bw + tw[v]; r[v] = 0.f; }
      const int* fx = tab + p.free_off;
      const int* fw = fx + p.tab_total;
      for (int q = 0; q < p.n_free; ++q) {
        const int dx = fx[q], dw = fw[q];
#pragma unroll
        for (int v = 0; v < V; ++v) r[v] = fmaf(load_one<IBF>(X, ox[v] + dx), load_one<IBF>(Wt, ow[v] + dw), r[v]);
      }
    }
    store_run<V, OBF>(out, run * V, r);
  }
}

// ---- gradients as gathers ------------------------------------------------------------------------------
// Backward-weight, and backward-data of views that are not one-to-one (an Expand sums, a Stride leaves gaps):
//   target[offT(i)] = sum over the other iterators of G[o] * other[offO(i)],   T, O = (W, X) or (X, W)
// over all iterators i = output axes and Reduce iterators.  The iterators whose T table varies ("carrying") pick
// the target element; the host has checked, by enumerating the tables, that every combination of their indices picks
// a different one (elements that none picks are zeroed first).  The remaining iterators are summed:
//   - long sums: a workgroup takes one combination and one slice of the remaining iterators flattened row-major;
//     threads keep private fp32 sums over runs along the innermost one, the workgroup adds them in a fixed tree, and
//     a second kernel adds the slices in order;
//   - short sums: a thread per combination walks the remaining iterators itself.
// No atomics either way, so the result does not depend on scheduling.
constexpr int kMaxIter = 2 * kMaxAxes;
struct ViewGradParams {
  ViewStream vs;
  int32_t tab_off[kMaxIter];
  int32_t tab_total, n_free, free_off;
  int32_t n_carry, n_rest;
  int32_t carry_axis[kMaxIter], rest_axis[kMaxIter];   // outermost first
  uint32_t rest_magic[kMaxIter];                       // division_magic(size) of the remaining iterators
  int32_t ostride[kMaxIter];                           // element stride in G (0 for a Reduce iterator)
  int32_t n_combo, n_splits;                           // carrying combinations; slices of a long sum (0: short sums)
  int32_t run;                                         // adjacent indices of the innermost remaining iterator per thread and step: 4 or 1
  int32_t zero_first;                                  // some target elements are picked by no combination
  int64_t total_rest, chunk;                           // runs over the remaining iterators (long sums) or their points (short); per slice
  int64_t target_elems;
};

struct GradBase { int g, o, t; };

// Offsets of carrying combination `combo`: in G, in the other operand, in the target (with the constant entries of
// the remaining iterators' target tables).
template <bool TO_X>
__device__ __forceinline__ GradBase grad_base(const ViewGradParams& p, const int* tab, int combo) {
  const int* tabT = TO_X ? tab : tab + p.tab_total;
  const int* tabO = TO_X ? tab + p.tab_total : tab;
  GradBase b{0, 0, 0};
  int rest = combo;
  for (int j = p.n_carry - 1; j >= 0; --j) {
    const int axis = p.carry_axis[j], sz = p.vs.size[axis], d = rest % sz;
    rest /= sz;
    b.g += d * p.ostride[axis];
    b.o += tabO[p.tab_off[axis] + d];
    b.t += tabT[p.tab_off[axis] + d];
  }
  for (int j = 0; j < p.n_rest; ++j) b.t += tabT[p.tab_off[p.rest_axis[j]]];
  return b;
}

template <bool OBF>
__device__ __forceinline__ void store_target(void* base, int64_t off, float v) {
  if constexpr (OBF) static_cast<uint16_t*>(base)[off] = (uint16_t)pack_bf16x2(v, 0.f);
  else static_cast<float*>(base)[off] = v;
}

template <bool IBF, bool TO_X>
__global__ __launch_bounds__(kThreads) void view_grad_long(const ViewGradParams p, const void* __restrict__ G,
                                                           const void* __restrict__ other, double* __restrict__ partial,
                                                           int* __restrict__ t_index) {
  extern __shared__ __align__(16) int tab[];
  __shared__ double wave_sum[kThreads / 64];
  const ViewStream& vs = p.vs;
  build_tables(vs, p.tab_off, p.free_off, p.n_free, p.tab_total, tab);
  const int* tabO = TO_X ? tab + p.tab_total : tab;
  const int combo = blockIdx.x / p.n_splits, slice = blockIdx.x - combo * p.n_splits;
  const GradBase b0 = grad_base<TO_X>(p, tab, combo);
  const int64_t begin = slice * p.chunk, end = min(p.total_rest, begin + p.chunk);
  // Sums run in fp64: a target element may be ONE sum over millions of products of either sign, whose fp32 partial
  // sums would lose, by cancellation, what a relative bar on the result demands; the loads bound these kernels, not
  // the arithmetic.
  double acc = 0.0;
  auto walk = [&](auto run_c) {
    constexpr int R = decltype(run_c)::value;
    const int inner = p.rest_axis[p.n_rest - 1];
    const uint32_t inner_runs = (uint32_t)vs.size[inner] / R;
    const int* to_inner = tabO + p.tab_off[inner];
    for (int64_t idx = begin + threadIdx.x; idx < end; idx += kThreads) {
      uint32_t rest = (uint32_t)idx;
      const uint32_t q0 = div_magic(rest, inner_runs, p.rest_magic[p.n_rest - 1]);
      const int d0 = (int)(rest - q0 * inner_runs) * R;
      rest = q0;
      int go = b0.g + d0 * p.ostride[inner], oo = b0.o;
      for (int j = p.n_rest - 2; j >= 0; --j) {
        const int axis = p.rest_axis[j];
        const uint32_t sz = (uint32_t)vs.size[axis];
        const uint32_t q = div_magic(rest, sz, p.rest_magic[j]);
        const int d = (int)(rest - q * sz);
        rest = q;
        go += d * p.ostride[axis];
        oo += tabO[p.tab_off[axis] + d];
      }
      float g[R], x[R];
#pragma unroll
      for (int k = 0; k < R; ++k) {
        g[k] = load_one<IBF>(G, go + k * p.ostride[inner]);
        x[k] = load_one<IBF>(other, oo + to_inner[d0 + k]);
      }
#pragma unroll
      for (int k = 0; k < R; ++k) acc = fma((double)g[k], (double)x[k], acc);
    }
  };
  if (p.run == 4) walk(std::integral_constant<int, 4>{});
  else walk(std::integral_constant<int, 1>{});
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) acc += __shfl_down(acc, d, 64);
  if ((threadIdx.x & 63) == 0) wave_sum[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = wave_sum[0];
    for (int w = 1; w < kThreads / 64; ++w) t += wave_sum[w];
    partial[blockIdx.x] = t;
    if (slice == 0) t_index[combo] = b0.t;
  }
}

template <bool OBF>
__global__ __launch_bounds__(kThreads) void view_grad_sum(const double* __restrict__ partial, const int* __restrict__ t_index,
                                                          void* __restrict__ target, int n_combo, int n_splits) {
  const int combo = blockIdx.x * kThreads + threadIdx.x;
  if (combo >= n_combo) return;
  double t = partial[(int64_t)combo * n_splits];
  for (int s = 1; s < n_splits; ++s) t += partial[(int64_t)combo * n_splits + s];
  store_target<OBF>(target, t_index[combo], (float)t);
}

template <bool IBF, bool OBF, bool TO_X>
__global__ __launch_bounds__(kThreads) void view_grad_short(const ViewGradParams p, const void* __restrict__ G,
                                                            const void* __restrict__ other, void* __restrict__ target) {
  extern __shared__ __align__(16) int tab[];
  const ViewStream& vs = p.vs;
  build_tables(vs, p.tab_off, p.free_off, p.n_free, p.tab_total, tab);
  const int* tabO = TO_X ? tab + p.tab_total : tab;
  const int64_t combo = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (combo >= p.n_combo) return;
  const GradBase b0 = grad_base<TO_X>(p, tab, (int)combo);
  double acc = 0.0;
  for (uint32_t idx = 0; idx < (uint32_t)p.total_rest; ++idx) {
    uint32_t rest = idx;
    int go = b0.g, oo = b0.o;
    for (int j = p.n_rest - 1; j >= 0; --j) {
      const int axis = p.rest_axis[j];
      const uint32_t sz = (uint32_t)vs.size[axis];
      const uint32_t q = div_magic(rest, sz, p.rest_magic[j]);
      const int d = (int)(rest - q * sz);
      rest = q;
      go += d * p.ostride[axis];
      oo += tabO[p.tab_off[axis] + d];
    }
    acc = fma((double)load_one<IBF>(G, go), (double)load_one<IBF>(other, oo), acc);
  }
  store_target<OBF>(target, b0.t, (float)acc);
}

// zeroes `bytes` bytes (a multiple of 2; dst is 4-byte aligned)
__global__ __launch_bounds__(kThreads) void view_grad_zero(uint32_t* __restrict__ dst, int64_t bytes) {
  const int64_t words = bytes >> 2;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < words; i += (int64_t)gridDim.x * kThreads) dst[i] = 0u;
  if ((bytes & 2) && blockIdx.x == 0 && threadIdx.x == 0) reinterpret_cast<uint16_t*>(dst)[bytes / 2 - 1] = 0;
}

constexpr int64_t kLongSum = 1024;       // remaining points from which a workgroup, not a thread, takes a combination

bool fill_grad(const syno_plan* plan, bool to_x, ViewGradParams& p) {
  p = ViewGradParams{};
  p.vs = plan->view;
  const ViewStream& vs = p.vs;
  p.target_elems = to_x ? plan->x_elems : plan->w_elems;
  if (plan->out_elems >= (int64_t(1) << 31) || plan->x_elems >= (int64_t(1) << 31) || plan->w_elems >= (int64_t(1) << 31)) return false;
  const int n_iter = vs.n_axes + vs.n_red;
  int total = 0;
  p.n_free = 1;
  for (int i = 0; i < n_iter; ++i) {
    p.tab_off[i] = total;
    total += vs.size[i];
    if (i >= vs.n_axes) p.n_free *= vs.size[i];
  }
  p.free_off = total;
  total += p.n_free;
  p.tab_total = total;
  if (total <= 0 || (size_t)total * 8 > 48 * 1024) return false;
  int64_t stride = 1;
  for (int i = vs.n_axes - 1; i >= 0; --i) { p.ostride[i] = (int32_t)stride; stride *= vs.size[i]; }
  // carrying iterators: those whose target table is not constant
  const int comp = to_x ? 0 : 1;
  int64_t n_combo = 1;
  p.total_rest = 1;
  int base = 0;
  std::vector<std::vector<int>> ttab;
  for (int i = 0; i < n_iter; ++i) {
    std::vector<int> col((size_t)vs.size[i]);
    bool varies = false;
    for (int o = 0; o < vs.size[i]; ++o) {
      int off[2];
      table_entry(vs, i, o, off);
      col[(size_t)o] = off[comp];
      varies |= off[comp] != col[0];
    }
    if (varies) {
      p.carry_axis[p.n_carry++] = i;
      n_combo *= vs.size[i];
      ttab.push_back(std::move(col));
    } else {
      base += col[0];
      p.rest_magic[p.n_rest] = division_magic(vs.size[i]);
      p.rest_axis[p.n_rest++] = i;
      p.total_rest *= vs.size[i];
    }
    if (n_combo > (int64_t(1) << 22) || p.total_rest >= (int64_t(1) << 31)) return false;   // (the check below enumerates them)
  }
  if (n_combo > p.target_elems || p.target_elems > (int64_t(1) << 26)) return false;   // (the check keeps a byte per target element)
  p.n_combo = (int32_t)n_combo;
  // every combination its own target element
  {
    std::vector<char> seen((size_t)p.target_elems, 0);
    for (int64_t combo = 0; combo < n_combo; ++combo) {
      int64_t rest = combo, t = base;
      for (int j = p.n_carry - 1; j >= 0; --j) { const int sz = vs.size[p.carry_axis[j]]; t += ttab[(size_t)j][(size_t)(rest % sz)]; rest /= sz; }
      if (t < 0 || t >= p.target_elems || seen[(size_t)t]) return false;
      seen[(size_t)t] = 1;
    }
  }
  p.zero_first = n_combo < p.target_elems ? 1 : 0;
  p.run = 1;
  if (p.total_rest >= kLongSum) {
    // a thread takes 4 adjacent indices of the innermost remaining iterator per step where that divides it
    const int inner = p.rest_axis[p.n_rest - 1];
    p.run = vs.size[inner] % 4 == 0 ? 4 : 1;
    p.rest_magic[p.n_rest - 1] = division_magic(vs.size[inner] / p.run);
    p.total_rest /= p.run;
    // about 2048 workgroups, each with at least a few thousand products
    const int64_t splits = std::max<int64_t>(1, std::min<int64_t>(2048 / n_combo, p.total_rest * p.run / 4096));
    p.chunk = (p.total_rest + splits - 1) / splits;
    p.n_splits = (int32_t)((p.total_rest + p.chunk - 1) / p.chunk);
    if ((int64_t)p.n_combo * p.n_splits >= (int64_t(1) << 31)) return false;
  }
  return true;
}

size_t grad_partial_bytes(const ViewGradParams& p) { return (((size_t)p.n_combo * p.n_splits * 8) + 255) & ~(size_t)255; }

template <bool IBF, bool OBF, bool SCATTER>
void launch_typed(const ViewParams& p, int V, size_t lds, const void* X, const void* W, void* out, hipStream_t s) {
  const int64_t blocks = (p.n_runs + kThreads - 1) / kThreads;
  const dim3 grid((unsigned)(blocks < p.max_blocks ? blocks : p.max_blocks));
  if (V == 4) hipLaunchKernelGGL((view_stream<4, IBF, OBF, SCATTER>), grid, dim3(kThreads), lds, s, p, X, W, out);
  else hipLaunchKernelGGL((view_stream<1, IBF, OBF, SCATTER>), grid, dim3(kThreads), lds, s, p, X, W, out);
}

template <bool SCATTER>
void launch_dtype(const syno_plan* plan, const ViewParams& p, int V, size_t lds, const void* A, const void* B, void* out,
                  hipStream_t s) {
  const bool ibf = plan->in_dtype == SYNO_BF16, obf = plan->out_dtype == SYNO_BF16;
  if (ibf && obf) launch_typed<true, true, SCATTER>(p, V, lds, A, B, out, s);
  else if (ibf) launch_typed<true, false, SCATTER>(p, V, lds, A, B, out, s);
  else launch_typed<false, false, SCATTER>(p, V, lds, A, B, out, s);
}

int run_width(const syno_plan* plan) {
  return plan->view.size[plan->view.n_axes - 1] % 4 == 0 ? 4 : 1;
}

// The magic for the innermost axis divides by its count of runs, not by its size.
bool fill(const syno_plan* plan, ViewParams& p) {
  p = ViewParams{};
  p.vs = plan->view;
  const int V = run_width(plan);
  int total = 0;
  p.n_free = 1;
  for (int i = 0; i < p.vs.n_axes + p.vs.n_red; ++i) {
    p.tab_off[i] = total;
    total += p.vs.size[i];
    if (i < p.vs.n_axes) p.magic[i] = division_magic(p.vs.size[i]);
    else p.n_free *= p.vs.size[i];
  }
  const int last = p.vs.n_axes - 1;
  p.magic[last] = division_magic(p.vs.size[last] / V);
  p.free_off = total;
  total += p.n_free;
  p.tab_total = total;
  p.n_runs = plan->out_elems / V;
  p.scratch_off = (2 * total + 3) & ~3;
  // eight workgroups per compute unit is what the registers allow to be resident
  p.max_blocks = plan->opt.view_workgroups > 0 ? plan->opt.view_workgroups : 256 * 8;
  return total > 0 && (size_t)total * 8 <= 48 * 1024 && p.n_runs < (int64_t(1) << 31);
}

}  // namespace

// Forward of every separable gather; backward-data where the view is one-to-one (a scatter of the same tables).
bool view_supports(const syno_plan* plan, int which) {
  if (!plan->pure_view) return false;
  if (plan->in_dtype == SYNO_F32 && plan->out_dtype != SYNO_F32) return false;
  if (which == SYNO_BWD_WEIGHT || (which == SYNO_BWD_DATA && !plan->view.one_to_one)) {
    ViewGradParams d;
    return fill_grad(plan, which == SYNO_BWD_DATA, d);
  }
  ViewParams p;
  return fill(plan, p);
}

void view_configure(syno_plan* plan, int which) {
  Launch& L = plan->launch[which];
  if (which == SYNO_BWD_WEIGHT || (which == SYNO_BWD_DATA && !plan->view.one_to_one)) {
    ViewGradParams d;
    static_assert(sizeof(ViewGradParams) <= sizeof(L.params), "parameter record does not fit");
    L.params_ready = fill_grad(plan, which == SYNO_BWD_DATA, d);
    memcpy(L.params, &d, sizeof d);
    // long sums: slice sums, then the target index of every combination
    L.workspace = d.n_splits > 0 ? grad_partial_bytes(d) + (size_t)d.n_combo * 4 : 0;
    return;
  }
  ViewParams p;
  static_assert(sizeof(ViewParams) <= sizeof(L.params), "parameter record does not fit");
  L.params_ready = fill(plan, p);
  memcpy(L.params, &p, sizeof p);
  L.workspace = 0;
}

std::string view_describe(const syno_plan* plan, int which) {
  if (!plan->launch[which].params_ready) return "unconfigured";
  if (which == SYNO_FWD) return "stream";
  if (which == SYNO_BWD_DATA && plan->view.one_to_one) return "scatter";
  ViewGradParams d;
  memcpy(&d, plan->launch[which].params, sizeof d);
  std::string r = "gather targets=" + std::to_string(d.n_combo) + " products/target=" + std::to_string(d.total_rest * d.run);
  r += d.n_splits > 0 ? " slices=" + std::to_string(d.n_splits) : std::string(" thread-per-target");
  if (d.zero_first) r += " zero-filled-first";
  return r;
}

// forward: A = X, B = W, out = result; backward-data: A = G, B = W, out = dX; backward-weight: A = G, B = X, out = dW
syno_status launch_view(const syno_plan* plan, int which, const void* A, const void* B, void* out, void* ws,
                        hipStream_t stream) {
  if (!plan->launch[which].params_ready) return SYNO_ERR_UNSUPPORTED;
  if (which == SYNO_BWD_WEIGHT || (which == SYNO_BWD_DATA && !plan->view.one_to_one)) {
    ViewGradParams d;
    memcpy(&d, plan->launch[which].params, sizeof d);
    const bool to_x = which == SYNO_BWD_DATA, ibf = plan->in_dtype == SYNO_BF16;
    const bool obf = to_x && plan->out_dtype == SYNO_BF16;          // (dW is always fp32)
    const size_t lds = (size_t)d.tab_total * 8;
    if (d.zero_first) {
      const int64_t bytes = d.target_elems * (obf ? 2 : 4), words = (bytes + 3) / 4;
      hipLaunchKernelGGL(view_grad_zero, dim3((unsigned)std::min<int64_t>((words + kThreads - 1) / kThreads, 2048)), dim3(kThreads),
                         0, stream, static_cast<uint32_t*>(out), bytes);
    }
    auto pick = [&](auto long_f32x, auto long_bfx, auto long_f32w, auto long_bfw) {
      return to_x ? (ibf ? long_bfx : long_f32x) : (ibf ? long_bfw : long_f32w);
    };
    if (d.n_splits > 0) {
      if (!ws) return SYNO_ERR_WORKSPACE;
      double* partial = static_cast<double*>(ws);
      int* t_index = reinterpret_cast<int*>(static_cast<char*>(ws) + grad_partial_bytes(d));
      const dim3 grid((unsigned)(d.n_combo * d.n_splits));
      auto k = pick(view_grad_long<false, true>, view_grad_long<true, true>, view_grad_long<false, false>, view_grad_long<true, false>);
      hipLaunchKernelGGL(k, grid, dim3(kThreads), lds, stream, d, A, B, partial, t_index);
      const dim3 sgrid((unsigned)((d.n_combo + kThreads - 1) / kThreads));
      if (obf) hipLaunchKernelGGL(view_grad_sum<true>, sgrid, dim3(kThreads), 0, stream, partial, t_index, out, d.n_combo, d.n_splits);
      else hipLaunchKernelGGL(view_grad_sum<false>, sgrid, dim3(kThreads), 0, stream, partial, t_index, out, d.n_combo, d.n_splits);
    } else {
      const dim3 grid((unsigned)((d.n_combo + kThreads - 1) / kThreads));
      if (obf) {
        hipLaunchKernelGGL((view_grad_short<true, true, true>), grid, dim3(kThreads), lds, stream, d, A, B, out);
      } else {
        auto k = pick(view_grad_short<false, false, true>, view_grad_short<true, false, true>, view_grad_short<false, false, false>,
                      view_grad_short<true, false, false>);
        hipLaunchKernelGGL(k, grid, dim3(kThreads), lds, stream, d, A, B, out);
      }
    }
    return hipGetLastError() == hipSuccess ? SYNO_OK : SYNO_ERR_HIP;
  }
  ViewParams p;
  memcpy(&p, plan->launch[which].params, sizeof p);
  const int V = run_width(plan);
  // the two tables, then (runs of 4) three 256-entry exchange areas for each of the 4 waves
  const size_t lds = V == 4 ? (size_t)p.scratch_off * 4 + (kThreads / 64) * 3 * 256 * 4 : (size_t)p.tab_total * 8;
  if (which == SYNO_FWD) launch_dtype<false>(plan, p, V, lds, A, B, out, stream);
  else launch_dtype<true>(plan, p, V, lds, A, B, out, stream);
  return hipGetLastError() == hipSuccess ? SYNO_OK : SYNO_ERR_HIP;
}

}  // namespace syno
