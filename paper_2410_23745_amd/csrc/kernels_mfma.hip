// MFMA contraction family: convolution-like operators whose Reduce is a real dense contraction,
//   out[n, g*Og+o, h, w] = sum_{c,kh,kw} X[n, g*Cg+c, row(h,kh,g), w+kw-pw] * W[g,o,c,kh,kw]
// computed as an implicit GEMM per group: M = output pixels (n,h,w), N = output channels o,
// K = (c,kh,kw).  Nothing is materialised: Unfold's window, Shift's cyclic row offset and the
// zero padding are folded into how the input tile is gathered into LDS.
//
// One workgroup owns TR whole output rows (of one or several images) x BN output channels.  Per
// chunk of KC input channels it stages
//   - the input rows those output rows touch, each row into a "slot" of Wp = Wi+KW-1 pixels whose
//     edge pixels stay zero (the padding), rows outside the image left zero; pixels are stored
//     channel-innermost, CI channels = 16 bytes per pixel (4 fp32 or 8 bf16), so that an MFMA
//     operand fragment is one LDS read per lane and a window tap is a constant address offset
//     (kh*Wp + kw pixels);
//   - the BN x KC x KH x KW weight block (fp32: as it lies in memory; bf16: from a copy a small
//     kernel has re-ordered into [tap][o][c], because the bf16 MFMA wants 8 consecutive channels
//     per lane);
// then issues 16x16 MFMAs whose K-step is 4 (fp32) or 32 (bf16) consecutive channels at one tap.
//
// The backward-data contraction is the same computation with the roles of the two channel axes
// exchanged, the taps reversed and the row shift negated, so it runs through the same kernel on
// an adjoint parameter record.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <type_traits>

#include "conv_mfma.h"
#include "plan.h"

namespace syno {

namespace {

// bf16 only: W[g][o][c][kh][kw] (any strides) -> blocks [g][nb][chunk] of [tap][o_local][w_row] with the
// channel innermost; rows beyond Og / Cg and the row padding are zero.  One thread gathers the 8
// channels of one 16-byte piece.
__global__ __launch_bounds__(256) void pack_weight_bf16(const MfmaParams p, const uint16_t* __restrict__ Wt,
                                                        uint4* __restrict__ packed, int64_t pieces) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= pieces) return;
  const int KHW = p.KH * p.KW, row8 = p.w_row >> 3;
  // Adjacent threads take adjacent taps, then adjacent output channels, of one channel octet: for the adjoint of a
  // forward-layout weight (output channel stride KHW, tap stride -1) and for a matrix product's transposed operand
  // (output channel stride 1) each of the 8 element loads of a wave then covers one contiguous stretch of memory;
  // the 16-byte pieces are written wherever the block layout puts them.
  int64_t r = i;
  const int tap = (int)(r % KHW); r /= KHW;
  const int ol = (int)(r % p.BN); r /= p.BN;
  const int cq = (int)(r % row8); r /= row8;
  const int ch = (int)(r % p.n_chunks); r /= p.n_chunks;
  const int nb = (int)(r % p.n_nblocks);
  const int g = (int)(r / p.n_nblocks);
  const int o = nb * p.BN + ol, cl0 = cq * 8, c0 = ch * p.KC + cl0;
  const int kh = tap / p.KW, kw = tap - kh * p.KW;
  uint32_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    v[e] = 0;
    if (cl0 + e < p.KC && o < p.Og && c0 + e < p.Cg)
      v[e] = Wt[p.w_base + (int64_t)g * p.ws_g + (int64_t)o * p.ws_o + (int64_t)(c0 + e) * p.ws_c + kh * p.ws_kh +
                kw * p.ws_kw];
  }
  const int64_t dst = (((((int64_t)g * p.n_nblocks + nb) * p.n_chunks + ch) * KHW + tap) * p.BN + ol) * row8 + cq;
  packed[dst] = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
}

// fp32 backward-data: Wt[g][c][o][kh'][kw'] = W[g][o][c][KH-1-kh'][KW-1-kw'] (source strides ts_*), contiguous.
__global__ __launch_bounds__(256) void transpose_weight_f32(const MfmaParams p, const float* __restrict__ Wt,
                                                            float* __restrict__ out, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  // (in the adjoint record Og counts the forward input channels and Cg the forward output channels)
  int64_t r = i;
  const int kw = (int)(r % p.KW); r /= p.KW;
  const int kh = (int)(r % p.KH); r /= p.KH;
  const int o = (int)(r % p.Cg); r /= p.Cg;
  const int c = (int)(r % p.Og);
  const int g = (int)(r / p.Og);
  out[i] = Wt[(int64_t)g * p.ts_g + (int64_t)o * p.ts_o + (int64_t)c * p.ts_c + (p.KH - 1 - kh) * p.ts_kh +
              (p.KW - 1 - kw) * p.ts_kw];
}

// The same re-ordering for weights in the forward layout [g][o][c][T taps] (contiguous): a thread takes
// 8 channels x T taps of one output channel (T adjacent 16-byte loads), re-orders them in registers and
// writes one 16-byte piece per tap.  Threads beyond Og / Cg write the zero pieces of the padding.
template <int T>
__global__ __launch_bounds__(256) void pack_weight_bf16_fwd(const MfmaParams p, const uint16_t* __restrict__ Wt,
                                                            uint4* __restrict__ packed, int64_t threads) {
  typedef uint32_t u32x4_unaligned __attribute__((ext_vector_type(4), aligned(2)));
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= threads) return;
  const int oct_per_chunk = p.KC >> 3, octs = p.n_chunks * oct_per_chunk, rows = p.n_nblocks * p.BN;
  const int octet = (int)(i % octs);
  const int row = (int)((i / octs) % rows);
  const int g = (int)(i / ((int64_t)octs * rows));
  const int ch = octet / oct_per_chunk, cq = octet - ch * oct_per_chunk;
  const int nb = row / p.BN, ol = row - nb * p.BN;
  const bool live = row < p.Og && octet * 8 < p.Cg;
  uint32_t in[4 * T];
#pragma unroll
  for (int q = 0; q < T; ++q) {
    u32x4_unaligned v = {0, 0, 0, 0};
    if (live)
      v = *reinterpret_cast<const u32x4_unaligned*>(Wt + (int64_t)g * p.ws_g + (int64_t)row * p.ws_o + octet * 8 * T + q * 8);
    in[4 * q + 0] = v[0]; in[4 * q + 1] = v[1]; in[4 * q + 2] = v[2]; in[4 * q + 3] = v[3];
  }
  uint4* block = packed + (((int64_t)(g * p.n_nblocks + nb) * p.n_chunks + ch) * p.w_block >> 3);
  const int row8 = p.w_row >> 3;
#pragma unroll
  for (int tap = 0; tap < T; ++tap) {
    uint32_t d[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const int e0 = (2 * h) * T + tap, e1 = (2 * h + 1) * T + tap;
      const uint32_t sel = ((e0 & 1) ? 0x0302u : 0x0100u) | ((e1 & 1) ? 0x07060000u : 0x05040000u);
      d[h] = __builtin_amdgcn_perm(in[e1 >> 1], in[e0 >> 1], sel);
    }
    block[(tap * p.BN + ol) * row8 + cq] = make_uint4(d[0], d[1], d[2], d[3]);
  }
}

// dst[c][r] = src[r][c], 32 x 32 tiles through LDS so that both sides move whole rows of a tile
template <class T>
__global__ __launch_bounds__(256) void transpose_2d(const T* __restrict__ src, T* __restrict__ dst, int rows, int cols) {
  __shared__ T tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = r0 + ty + 8 * i, c = c0 + tx;
    if (r < rows && c < cols) tile[ty + 8 * i][tx] = src[(int64_t)r * cols + c];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = c0 + ty + 8 * i, r = r0 + tx;
    if (r < rows && c < cols) dst[(int64_t)c * rows + r] = tile[tx][ty + 8 * i];
  }
}

// out[i] = parts[0][i] + parts[1][i] + ... (k partial results `stride` elements apart, added in this order)
__global__ __launch_bounds__(256) void sum_split_results(const float* __restrict__ parts, float* __restrict__ out,
                                                         int64_t n, int k, int64_t stride) {
  const int64_t step = (int64_t)gridDim.x * 256;
  if ((n & 3) == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < (n >> 2); i += step) {
      float4 a = reinterpret_cast<const float4*>(parts)[i];
      for (int j = 1; j < k; ++j) {
        const float4 b = reinterpret_cast<const float4*>(parts + j * stride)[i];
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
      }
      reinterpret_cast<float4*>(out)[i] = a;
    }
  } else {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += step) {
      float a = parts[i];
      for (int j = 1; j < k; ++j) a += parts[j * stride + i];
      out[i] = a;
    }
  }
}

// Gradients of a convolution with stride s through its phase planes (the s*s sub-images X[.., s*h'+a, s*w'+b] taken as
// s*s*C channels, on which the window moves with stride 1).  Tap kh of the strided window reads phase a = (kh-p) mod s
// at row offset dh = floor((kh-p)/s), which is tap dh+1 of a 3-wide stride-1 window with pad 1 (or the only tap of a
// 1-wide one).  The two kernels move weights between the two forms; `taps` = s*dh+a+p for every (a, tap) is recomputed
// from the record.
struct PhaseParams {
  int32_t O, C, K, s, p, window;
  int32_t ws_o, ws_c, ws_kh, ws_kw;
};

__device__ __forceinline__ int floor_div(int a, int b) { return (a >= 0 ? a : a - b + 1) / b; }

// one thread per element of dW
__global__ __launch_bounds__(256) void phase_weight_gather(const PhaseParams q, const float* __restrict__ dWp,
                                                           float* __restrict__ dW) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= q.O * q.C * q.K * q.K) return;
  int r = i;
  const int kw = r % q.K; r /= q.K;
  const int kh = r % q.K; r /= q.K;
  const int c = r % q.C;
  const int o = r / q.C;
  const int dh = floor_div(kh - q.p, q.s), a = kh - q.p - q.s * dh;
  const int dw = floor_div(kw - q.p, q.s), b = kw - q.p - q.s * dw;
  const int th = q.window == 3 ? dh + 1 : 0, tw = q.window == 3 ? dw + 1 : 0;
  const int cp = (c * q.s + a) * q.s + b;
  dW[(int64_t)o * q.ws_o + (int64_t)c * q.ws_c + kh * q.ws_kh + kw * q.ws_kw] =
      dWp[(((int64_t)o * q.C * q.s * q.s + cp) * q.window + th) * q.window + tw];
}

// one thread per element of Wpp
template <class T>
__global__ __launch_bounds__(256) void phase_weight_build(const PhaseParams q, const T* __restrict__ W, T* __restrict__ Wpp) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  const int CP = q.C * q.s * q.s;
  if (i >= CP * q.O * q.window * q.window) return;
  int r = i;
  const int tw = r % q.window; r /= q.window;
  const int th = r % q.window; r /= q.window;
  const int o = r % q.O;
  const int cp = r / q.O;
  const int b = cp % q.s, a = (cp / q.s) % q.s, c = cp / (q.s * q.s);
  const int dh = q.window == 3 ? th - 1 : 0, dw = q.window == 3 ? tw - 1 : 0;
  const int kh = a + q.p - q.s * dh, kw = b + q.p - q.s * dw;
  T v = 0;
  if (kh >= 0 && kh < q.K && kw >= 0 && kw < q.K)
    v = W[(int64_t)o * q.ws_o + (int64_t)c * q.ws_c + kh * q.ws_kh + kw * q.ws_kw];
  Wpp[i] = v;
}

// ---------------------------------------------------------------------------------------------
// Host side: tile choice and launch
// ---------------------------------------------------------------------------------------------
constexpr int kNumCU = 256;

int num_variants(bool bf) { return bf ? kNumBf16Variants : kNumF32Variants; }
const Variant& variant_of(bool bf, int vi) { return bf ? kBf16Variants[vi] : kF32Variants[vi]; }

// most images a run of TR consecutive output rows can touch (blocks start at multiples of TR)
int images_spanned(int TR, int Ho) {
  if (Ho % TR == 0) return 1;
  if (TR % Ho == 0) return TR / Ho;
  return (TR + Ho - 2) / Ho + 1;
}

// Row slots a block of TR output rows needs: a run of r rows of one image takes (r-1)*sh + KH consecutive input rows
int row_slots(const ConvLike& c, int sh, int TR) {
  if (c.h_wrap) return TR;
  const int per_image = c.KH - sh;      // (may be negative: a 1x1 window under a Stride)
  return TR * sh + per_image * (per_image >= 0 ? images_spanned(TR, c.Ho) : 1);
}

// LDS weight row pitch (in dwords) >= need such that the 64 lanes of a B-fragment read (16 rows x 4
// channel steps of `kstep` dwords) fall into distinct banks where possible.
int pick_w_row(int need, int kstep, int multiple_of) {
  int best = need, best_conf = 1 << 30;
  for (int r = (need + multiple_of - 1) / multiple_of * multiple_of; r < need + 128; r += multiple_of) {
    int cnt[64] = {};
    int conf = 0;
    for (int n = 0; n < 16; ++n)
      for (int k = 0; k < 4; ++k) conf = std::max(conf, ++cnt[(n * r + k * kstep) & 63]);
    if (conf < best_conf) { best_conf = conf; best = r; }
    if (conf == 1) break;
  }
  return best;
}

// bf16 tile variants whose backward-data instantiation reads forward-layout 3x3 weights itself (the others pack)
bool bf16_adjoint_direct(int vi) { return vi == 1 || vi == 8 || vi == 9; }

// Parameter record of contraction `which` (forward, or backward-data as its adjoint) for tile variant vi
// and TR output rows per block.  False when the combination does not fit the kernel's static limits.
bool fill_params(const syno_plan* plan, int which, int vi, int TR, MfmaParams& p, int ksplit = 1) {
  const ConvLike& c = plan->conv;
  const bool bf = plan->in_dtype == SYNO_BF16;
  if (vi < 0 || vi >= num_variants(bf) || TR < 1) return false;
  // the kernel addresses its source tensor with 32-bit byte offsets
  if ((which == SYNO_FWD ? plan->x_elems : plan->out_elems) * (bf ? 2 : 4) >= (1ll << 32)) return false;
  const Variant& v = variant_of(bf, vi);
  p = MfmaParams{};
  p.G = c.G; p.Ho = c.Ho; p.Wo = c.Wo; p.Hi = c.Hi; p.Wi = c.Wi;
  p.KH = c.KH; p.KW = c.KW;
  p.rows_total = c.N * c.Ho;
  p.h_wrap = c.h_wrap;
  p.sh = p.sw = 1;
  const int plane = c.Hi * c.Wi;
  if (which == SYNO_FWD) {
    p.Og = c.Og; p.Cg = c.Cg; p.ph = c.ph; p.pw = c.pw;
    p.sh = c.sh; p.sw = c.sw;         // (only forward takes a Stride below the window; its result plane is Ho x Wo)
    p.h_shift = c.h_shift; p.h_shift_g = c.h_shift_g;
    p.xs_c = plane; p.xs_n = c.G * c.Cg * plane;
    p.os_o = c.Ho * c.Wo; p.os_n = c.G * c.Og * c.Ho * c.Wo;
    p.ws_g = c.ws_g; p.ws_o = c.ws_o; p.ws_c = c.ws_c; p.ws_kh = c.ws_kh; p.ws_kw = c.ws_kw; p.w_base = 0;
  } else {
    // dX[n,g*Cg+c,y,x] = sum_{o,kh',kw'} G[n,g*Og+o, y+kh'-(KH-1-ph), x+kw'-(KW-1-pw)] * W[g,o,c,KH-1-kh',KW-1-kw']
    p.Og = c.Cg; p.Cg = c.Og; p.ph = c.KH - 1 - c.ph; p.pw = c.KW - 1 - c.pw;
    p.h_shift = (c.Hi - c.h_shift % c.Hi) % c.Hi; p.h_shift_g = (c.Hi - c.h_shift_g % c.Hi) % c.Hi;
    p.xs_c = plane; p.xs_n = c.G * c.Og * plane;
    p.os_o = plane; p.os_n = c.G * c.Cg * plane;
    p.ws_g = c.ws_g; p.ws_o = c.ws_c; p.ws_c = c.ws_o; p.ws_kh = -c.ws_kh; p.ws_kw = -c.ws_kw;
    p.w_base = (c.KH - 1) * c.ws_kh + (c.KW - 1) * c.ws_kw;
    if (!bf) {
      // fp32: a small kernel first writes the adjoint's weights [g][c][o][reversed taps] contiguously into the
      // workspace, so that the contraction stages them in 16-byte pieces like forward weights
      p.wt = 1;
      p.ts_g = c.ws_g; p.ts_o = c.ws_o; p.ts_c = c.ws_c; p.ts_kh = c.ws_kh; p.ts_kw = c.ws_kw;
      p.ws_g = c.Cg * c.Og * c.KH * c.KW; p.ws_o = c.Og * c.KH * c.KW; p.ws_c = c.KH * c.KW; p.ws_kh = c.KW; p.ws_kw = 1;
      p.w_base = 0;
    }
  }
  p.TR = TR;
  p.BN = v.BN();
  const int KHW = c.KH * c.KW;
  const int CI = bf ? 8 : 4;
  if (bf) {
    p.KC = v.KC;
    if (v.one && p.Cg > p.KC) return false;
    if (v.BN() == 128 && KHW != 1) return false;   // (the 128-channel variant is instantiated for 1x1 windows only)
    p.w_row = p.KC + 8;                          // elements; 80- and 144-byte rows keep B-fragment reads conflict free
    p.w_block = KHW * p.BN * p.w_row;
    // Forward-layout weights [o][c][taps] are read unpacked: by every variant when there are 9 taps, by the
    // single-chunk variant also with 3 or 1 (and through the adjoint for backward-data, marked by a negative count)
    const bool fwd_layout = (c.KW == 1 || c.ws_kw == 1) && (c.KH == 1 || c.ws_kh == c.KW) && c.ws_c == KHW;
    if (fwd_layout && (c.Cg & 7) == 0) {
      // (variant 0 is also instantiated for 3 taps: the 3x1 second stage of the paper's Operator 1 runs there)
      if (which == SYNO_FWD && (KHW == 9 || (v.one && (KHW == 1 || KHW == 3)) || (KHW == 3 && vi == 0))) p.wf = KHW;
      if (which == SYNO_BWD_DATA && v.one && (KHW == 1 || KHW == 3 || KHW == 9)) p.wf = -KHW;
    }
    // backward-data of a 3x3 window by the chunked variants instantiated for it: runs of 9 taps per (output channel,
    // channel) pair, the reduction (forward output channels) in whole octets, the source addressed in 32 bits
    if (fwd_layout && which == SYNO_BWD_DATA && !v.one && KHW == 9 && (c.Og & 7) == 0 && bf16_adjoint_direct(vi) &&
        c.ws_o == c.Cg * KHW && (int64_t)c.Og * c.ws_o < (1ll << 30))
      p.wf = -KHW;
    if (p.wf == 0 && (p.w_block >> 3) > v.WI * v.NT()) return false;
  } else if (v.wnat) {
    if ((c.KW > 1 && p.ws_kw != 1) || (c.KH > 1 && p.ws_kh != c.KW) || p.ws_c != KHW || (p.ws_o & 3) || (p.ws_g & 3))
      return false;
    p.KC = v.KC;
    while (p.KC > 8 && (p.Cg % p.KC != 0 || p.BN * p.KC * KHW > 4 * v.WI * v.NT() ||
                        (p.KC / CI) * row_slots(c, p.sh, TR) * ((c.Wi < 4) ? c.Wi : (c.Wi + 3) / 4) > v.XI * v.NT()))
      p.KC -= 8;
    if (p.Cg % p.KC != 0 || ((p.KC * KHW) & 3) || p.BN * p.KC * KHW > 4 * v.WI * v.NT()) return false;
    p.w_row = pick_w_row(p.KC * KHW, KHW, 4);
    // backward-data of a 3x3 window whose weights lie in the forward layout: no transposed copy, the kernel takes the
    // 9 taps of every (output channel, channel) pair as they lie and turns them round on the way into LDS
    if (which == SYNO_BWD_DATA && p.wt && KHW == 9 && c.ws_kw == 1 && c.ws_kh == c.KW && c.ws_c == KHW &&
        c.ws_o == c.Cg * KHW && ((p.BN * p.KC + v.NT() - 1) / v.NT()) * 9 <= 4 * v.WI) {
      p.wt = 0; p.wadj = 1;
      p.ws_g = c.ws_g; p.ws_o = KHW; p.ws_c = c.ws_o; p.ws_kh = c.KW; p.ws_kw = 1; p.w_base = 0;
    }
  } else {
    p.KC = v.KC;
    while (p.KC > 4 && (p.BN * p.KC * KHW > v.WI * v.NT())) p.KC -= 4;
    if (p.BN * p.KC * KHW > v.WI * v.NT()) return false;
    p.w_row = pick_w_row(p.KC * KHW, KHW, 1);
  }
  p.cgrps = p.KC / CI;
  p.n_chunks = (p.Cg + p.KC - 1) / p.KC;
  // three taps per row-step when the window is 3 wide and the row-steps still divide evenly among the K-split waves
  p.U = (!bf && c.KW == 3 && (p.cgrps * c.KH) % v.WK == 0) ? 3 : 1;   // (bf16 runs out of registers with 3)
  p.n_mblocks = (p.rows_total + TR - 1) / TR;
  p.n_nblocks = (p.Og + p.BN - 1) / p.BN;
  p.n_slots = row_slots(c, p.sh, TR);
  p.Wp = c.Wi + c.KW - 1;
  if ((TR * c.Wo + 15) / 16 > v.MT()) return false;
  p.vx = c.Wi < 4 ? 1 : 4;
  p.vpr = (c.Wi + p.vx - 1) / p.vx;
  if (p.cgrps * p.n_slots * p.vpr > v.XI * v.NT()) return false;
  const int x_bytes = p.cgrps * p.n_slots * p.Wp * 16;
  p.lds_w_off = x_bytes;
  const int w_bytes = bf ? p.w_block * 2 : p.BN * p.w_row * 4;
  p.lds_tab_off = p.lds_w_off + ((w_bytes + 15) & ~15);
  p.lds_bytes = p.lds_tab_off + ((p.n_slots * 4 + 15) & ~15);
  if (v.WK > 1) p.lds_bytes = std::max(p.lds_bytes, v.WM * v.WN * v.TM * v.TN * 1024);
  if (!bf && p.w_row * p.BN >= (1 << 20)) return false;
  auto magic = [](int64_t d) { return (uint32_t)(((1ull << 32) + d - 1) / std::max<int64_t>(d, 1)); };
  const int64_t per_cg = (int64_t)p.n_slots * p.vpr;
  const int64_t per_o = bf ? 1 : (v.wnat ? (p.KC * KHW) >> 2 : p.KC * KHW);
  // largest numerators: item indices (< XI*NT, WI*NT), pixels of a block (< 16*MT), output rows (< rows_total)
  const int64_t max_idx = (int64_t)std::max(v.XI, v.WI) * v.NT();
  if (max_idx * per_cg >= (1ll << 32) || max_idx * per_o >= (1ll << 32) || (int64_t)p.rows_total * c.Ho >= (1ll << 32))
    return false;
  p.m_wo = magic(c.Wo); p.m_ho = magic(c.Ho); p.m_vpr = magic(p.vpr); p.m_pcg = magic(per_cg);
  p.m_per_o = magic(per_o); p.m_khw = magic(KHW); p.m_kw = magic(c.KW);
  // workgroups that share an output tile and split the chunks: fp32 partial results, every range non-empty
  p.ksplit = 1; p.chunks_per_split = p.n_chunks; p.split_stride = 0;
  if (ksplit > 1) {
    const int64_t result = which == SYNO_FWD ? plan->out_elems : plan->x_elems;
    if (v.one || plan->out_dtype != SYNO_F32 || ksplit > p.n_chunks || result >= (1ll << 31) - 4) return false;
    p.chunks_per_split = (p.n_chunks + ksplit - 1) / ksplit;
    if ((int64_t)(ksplit - 1) * p.chunks_per_split >= p.n_chunks) return false;
    p.ksplit = ksplit;
    p.split_stride = (int32_t)((result + 3) & ~3ll);
  }
  // Which tiles share an XCD's L2: with the tiles of a plane dealt as xcd_m x xcd_n rectangles the XCDs together fetch
  // the source xcd_n times and the weights xcd_m times; take the split with the fewest bytes that divides both counts.
  // An XCD walks its rectangle either one row of tiles after the other, coming back to the same weight panels in each
  // row, or one panel after the other, coming back to the same source rows: unless the whole rectangle is resident at
  // once, the operand it comes back to has to stay in that XCD's L2 (4 MB, half of it left to the streaming one), or
  // every pass fetches it again.
  p.xcd_m = p.xcd_n = p.xcd_rows_first = 0;
  if (((int64_t)p.n_mblocks * p.n_nblocks) % 8 == 0) {
    const double esize = bf ? 2.0 : 4.0, fits = 2.0 * 1024 * 1024;
    const double src = esize * c.N * p.Cg * plane / p.ksplit, wts = esize * p.Og * p.Cg * KHW / p.ksplit;
    const int64_t resident = 32 * std::max(1, std::min(2, kMaxLdsBytes / std::max(p.lds_bytes, 1)));
    double fewest = 0;
    for (int a = 1; a <= 8; a *= 2) {
      const int b = 8 / a;
      if (p.n_mblocks % a != 0 || p.n_nblocks % b != 0) continue;
      const int64_t sm = p.n_mblocks / a, sn = p.n_nblocks / b;
      for (int rows_first = 0; rows_first < 2; ++rows_first) {
        double bytes = b * src + a * wts;
        if (sm * sn > resident) {
          if (!rows_first && wts / b > fits) bytes += a * wts * (sm - 1);
          if (rows_first && src / a > fits) bytes += b * src * (sn - 1);
        }
        if (p.xcd_m == 0 || bytes < fewest) { fewest = bytes; p.xcd_m = a; p.xcd_n = b; p.xcd_rows_first = rows_first; }
      }
    }
  }
  return p.lds_bytes <= kMaxLdsBytes;
}

// Estimated duration of the launch in SIMD cycles.  Row tiles are dealt evenly to the WM wave rows, wave
// widx runs on SIMD widx%4, a 16x16 MFMA occupies its SIMD's matrix pipe for 32 (fp32 K=4) or 16 (bf16
// K=32) cycles, and one k-step of a wave cannot finish faster than its LDS reads allow.  Staging, barriers
// and the prologue overlap with another resident workgroup's MFMAs only when more than one fits on a CU.
double tile_cost(const MfmaParams& p, const Variant& v, const ConvLike& c, bool bf) {
  const int64_t wgs = (int64_t)p.n_mblocks * p.n_nblocks * c.G * p.ksplit;
  const int MT = (std::min(p.TR, p.rows_total) * c.Wo + 15) / 16;
  const int base = MT / v.WM, extra = MT % v.WM;
  const double mfma_cycles = bf ? 16.0 : 32.0, read_cycles = bf ? 16.0 : 8.0;
  // per k-step of the chunk: cycles of matrix pipe and of step latency each SIMD sees, averaged over the
  // waves that split the steps
  double simd_mfma[4] = {0, 0, 0, 0}, simd_lat[4] = {0, 0, 0, 0};
  for (int widx = 0; widx < v.WM * v.WN * v.WK; ++widx) {
    const int wtile = widx % (v.WM * v.WN);
    const int wk = widx / (v.WM * v.WN);
    const int wn = wtile / v.WM, wm = (wtile + wn + ((wk * v.WM * v.WN) >> 2)) % v.WM;
    const int tiles = base + (wm < extra ? 1 : 0);
    if (!tiles) continue;
    simd_mfma[widx & 3] += mfma_cycles * tiles * v.TN / v.WK;
    // a wave's step: address arithmetic, LDS round trip, then its MFMAs issue
    simd_lat[widx & 3] += (200.0 + read_cycles * (tiles + v.TN)) / v.WK;
  }
  double step = 0;
  for (int s = 0; s < 4; ++s) step = std::max(step, std::max(simd_mfma[s], 0.5 * simd_lat[s] + 0.5 * simd_mfma[s]));
  const double steps = (double)p.chunks_per_split * (p.cgrps / (bf ? 4 : 1)) * c.KH * c.KW;
  const double overhead = p.chunks_per_split * 5000.0 + 6000.0 + (v.WK - 1) * 1500.0;
  // the second kernel of a split: its launch, and the partial results written and read back at about 3 TB/s
  const double split_cost = p.ksplit > 1 ? 10000.0 + (2.0 * p.ksplit + 1.0) * p.split_stride * 4.0 / 3.0e12 * 2.4e9 : 0.0;
  // 8 waves of up to 256 VGPRs fill a CU's register file; 4-wave workgroups fit twice
  const int resident = (v.NT() <= 256 && p.lds_bytes <= kMaxLdsBytes / 2) ? 2 : 1;
  const double per_cu_wgs = std::ceil((double)wgs / kNumCU);
  return per_cu_wgs * steps * step + std::ceil(per_cu_wgs / resident) * overhead + split_cost;
}

size_t packed_weight_bytes(const MfmaParams& p) {
  return (size_t)p.G * p.n_nblocks * p.n_chunks * p.w_block * 2;
}

// head of the workspace: the re-ordered weights (rounded up so that the partial results behind it stay aligned)
size_t weight_workspace_bytes(const MfmaParams& p, bool bf) {
  const size_t n = bf ? (p.wf == 0 ? packed_weight_bytes(p) : 0) : (p.wt ? (size_t)p.G * p.Og * p.Cg * p.KH * p.KW * 4 : 0);
  return (n + 255) & ~(size_t)255;
}

}  // namespace

bool mfma_supports(const syno_plan* p, int which) {
  if (!p->conv_like || which == SYNO_BWD_WEIGHT) return false;
  if (p->in_dtype == SYNO_F32 && p->out_dtype != SYNO_F32) return false;   // not instantiated
  const ConvLike& c = p->conv;
  if (c.w_wrap) return false;
  if (c.h_wrap && c.KH != 1) return false;
  if (c.sh != 1 || c.sw != 1) {
    // a Stride below the window: forward only (its adjoint scatters), rows not cyclic, every tap inside the padded row
    if (which != SYNO_FWD || c.h_wrap || c.sh < 1 || c.sw < 1 || c.sh > 4 || c.sw > 4) return false;
    if ((c.Wo - 1) * c.sw >= c.Wi || (c.Ho - 1) * c.sh - c.ph >= c.Hi) return false;
  } else if (c.Wi != c.Wo || c.Hi != c.Ho) {
    return false;
  }
  if (c.ph >= c.KH || c.pw >= c.KW) return false;
  if (c.Og == 1 && c.Cg == 1) return false;          // no contraction to speak of
  if (rows_supports(p, which)) return true;
  MfmaParams mp;
  for (int vi = 0; vi < num_variants(p->in_dtype == SYNO_BF16); ++vi)
    for (int TR = 1; TR <= c.N * c.Ho && TR * c.Wo <= 16 * 32; ++TR)
      if (fill_params(p, which, vi, TR, mp)) return true;
  return false;
}

void mfma_configure(syno_plan* plan, int which) {
  const ConvLike& c = plan->conv;
  const bool bf = plan->in_dtype == SYNO_BF16;
  // bf16 operators whose whole reduction fits LDS go to the row-streaming kernel (unless a tile variant is named)
  if (bf && plan->opt.mfma_variant <= 0 && rows_configure(plan, which)) return;
  double best = 1e300;
  int best_v = -1, best_tr = 0;
  MfmaParams mp;
  // the descriptor's options may name the tile variant and the rows per block (verification and tuning aid).
  // A reduction over thousands of channels whose tiles would leave compute units idle may be split over workgroups
  // (each still runs at least 32 chunks); the option names a split outright
  const int forced = plan->opt.mfma_splits > 0 ? plan->opt.mfma_splits : 0;
  const int splits[] = {1, 2, 3, 4, 6, 8};
  int best_ks = 1;
  if (plan->opt.mfma_variant > 0 && fill_params(plan, which, plan->opt.mfma_variant - 1, plan->opt.mfma_rows, mp, forced ? forced : 1)) {
    best_v = plan->opt.mfma_variant - 1; best_tr = plan->opt.mfma_rows; best_ks = forced ? forced : 1;
  }
  if (best_v < 0)
    for (int vi = 0; vi < num_variants(bf); ++vi)
      for (int TR = 1; TR <= c.N * c.Ho && TR * c.Wo <= 16 * 32; ++TR) {
        if (!fill_params(plan, which, vi, TR, mp)) continue;      // (a split only adds conditions)
        const int n_chunks = mp.n_chunks;
        for (int ks : splits) {
          const int k = forced ? forced : ks;
          if (!forced && k > 1 && n_chunks < 32 * k) break;
          if (k > 1 && !fill_params(plan, which, vi, TR, mp, k)) { if (forced) break; else continue; }
          const double cost = tile_cost(mp, variant_of(bf, vi), c, bf);
          if (cost < best) { best = cost; best_v = vi; best_tr = TR; best_ks = k; }
          if (forced) break;
        }
      }
  if (best_v < 0 && forced)      // (the named split does not fit this operator: the planner's own choice)
    for (int vi = 0; vi < num_variants(bf); ++vi)
      for (int TR = 1; TR <= c.N * c.Ho && TR * c.Wo <= 16 * 32; ++TR) {
        if (!fill_params(plan, which, vi, TR, mp)) continue;
        const double cost = tile_cost(mp, variant_of(bf, vi), c, bf);
        if (cost < best) { best = cost; best_v = vi; best_tr = TR; best_ks = 1; }
      }
  fill_params(plan, which, best_v, best_tr, mp, best_ks);
  if (plan->opt.mfma_taps == 1) mp.U = 1;     // (option: the one-tap-per-row-step instantiation)
  mp.probe_lo = (uint32_t)reinterpret_cast<uintptr_t>(plan->opt.clock_probe);
  mp.probe_hi = (uint32_t)(reinterpret_cast<uintptr_t>(plan->opt.clock_probe) >> 32);
  static_assert(sizeof(MfmaParams) <= sizeof(plan->launch[which].params), "parameter record does not fit");
  memcpy(plan->launch[which].params, &mp, sizeof mp);
  plan->launch[which].params_ready = true;
  plan->launch[which].variant = best_v * 4096 + best_tr;
  plan->launch[which].workspace = weight_workspace_bytes(mp, bf) + (mp.ksplit > 1 ? (size_t)mp.ksplit * mp.split_stride * 4 : 0);
}

std::string mfma_describe(const syno_plan* plan, int which) {
  if (plan->launch[which].variant == -1) return rows_describe(plan, which);
  const int vi = plan->launch[which].variant / 4096, TR = plan->launch[which].variant % 4096;
  MfmaParams p;
  if (!fill_params(plan, which, vi, TR, p)) return "unconfigured";
  const Variant& v = variant_of(plan->in_dtype == SYNO_BF16, vi);
  char b[256];
  memcpy(&p, plan->launch[which].params, sizeof p);
  snprintf(b, sizeof b, "variant=%d rows/block=%d BN=%d KC=%d taps/row-step=%d weights=%s waves=%dx%dx%d grid=%d lds=%dB slots=%d", vi, TR,
           v.BN(), p.KC, p.U, plan->in_dtype != SYNO_BF16 ? (p.wt ? "transposed-copy" : p.wadj ? "turned-while-staged" : "direct") : (p.wf ? "direct" : "packed"), v.WM, v.WN, v.WK, p.n_mblocks * p.n_nblocks * p.G * p.ksplit, p.lds_bytes, p.n_slots);
  std::string d = b;
  if (p.xcd_m > 0)
    d += " tiles-per-xcd=" + std::to_string(p.n_mblocks / p.xcd_m) + "x" + std::to_string(p.n_nblocks / p.xcd_n) +
         (p.xcd_rows_first ? "(rows first)" : "");
  if (p.ksplit > 1) d += " reduction-splits=" + std::to_string(p.ksplit);
  return d;
}

syno_status launch_mfma(const syno_plan* plan, int which, const void* A, const void* B, void* out, void* ws,
                        hipStream_t stream) {
  const int vi = plan->launch[which].variant / 4096;
  if (!plan->launch[which].params_ready) return SYNO_ERR_UNSUPPORTED;
  if (plan->launch[which].variant == -1) return launch_rows(plan, which, A, B, out, ws, stream);
  MfmaParams p;
  memcpy(&p, plan->launch[which].params, sizeof p);
  const bool obf = plan->out_dtype == SYNO_BF16;
  // a split reduction leaves its partial results behind the weights in the workspace
  void* const result = out;
  if (p.ksplit > 1) {
    if (!ws) return SYNO_ERR_WORKSPACE;
    out = static_cast<char*>(ws) + weight_workspace_bytes(p, plan->in_dtype == SYNO_BF16);
  }
  if (plan->in_dtype == SYNO_BF16) {
    const void* weights = B;
    if (p.wf == 0) {
      if (!ws) return SYNO_ERR_WORKSPACE;
      const ConvLike& c = plan->conv;
      const int KHW = c.KH * c.KW;
      const bool fwd_layout = which == SYNO_FWD && (c.KW == 1 || c.ws_kw == 1) && (c.KH == 1 || c.ws_kh == c.KW) &&
                              c.ws_c == KHW && (c.Cg & 7) == 0;
      const uint16_t* Wt = static_cast<const uint16_t*>(B);
      uint4* dst = static_cast<uint4*>(ws);
      const int64_t threads = (int64_t)p.G * p.n_nblocks * p.BN * p.n_chunks * (p.KC >> 3);
      const dim3 grid((unsigned)((threads + 255) / 256));
      if (fwd_layout && KHW == 9) hipLaunchKernelGGL(pack_weight_bf16_fwd<9>, grid, dim3(256), 0, stream, p, Wt, dst, threads);
      else if (fwd_layout && KHW == 3) hipLaunchKernelGGL(pack_weight_bf16_fwd<3>, grid, dim3(256), 0, stream, p, Wt, dst, threads);
      else if (fwd_layout && KHW == 1) hipLaunchKernelGGL(pack_weight_bf16_fwd<1>, grid, dim3(256), 0, stream, p, Wt, dst, threads);
      else {
        const int64_t pieces = (int64_t)packed_weight_bytes(p) / 16;
        hipLaunchKernelGGL(pack_weight_bf16, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, stream, p, Wt, dst, pieces);
      }
      weights = ws;
    }
    if (obf) launch_mfma_bf16_bf16out(vi, p, A, weights, out, stream);
    else launch_mfma_bf16_f32out(vi, p, A, weights, out, stream);
  } else {
    if (obf) return SYNO_ERR_UNSUPPORTED;
    const void* weights = B;
    if (p.wt) {
      if (!ws) return SYNO_ERR_WORKSPACE;
      const int64_t n = (int64_t)p.G * p.Og * p.Cg * p.KH * p.KW;
      // a 1x1 window over a contiguous [o][c] matrix is a plain transposition, which goes through LDS tiles
      const bool plain = p.G == 1 && p.KH * p.KW == 1 && p.ts_c == 1 && p.ts_o == p.Og;
      if (!plain || launch_transpose_2d(B, ws, p.Cg, p.Og, 4, stream) != SYNO_OK)
        hipLaunchKernelGGL(transpose_weight_f32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p,
                           static_cast<const float*>(B), static_cast<float*>(ws), n);
      weights = ws;
    }
    if (vi < 4) launch_mfma_f32_lo(vi, p, A, weights, out, stream);
    else launch_mfma_f32_hi(vi, p, A, weights, out, stream);
  }
  if (p.ksplit > 1) {
    const int64_t n = which == SYNO_FWD ? plan->out_elems : plan->x_elems;
    const int64_t blocks = std::min<int64_t>(((n + 3) / 4 + 255) / 256, 8 * kNumCU);
    hipLaunchKernelGGL(sum_split_results, dim3((unsigned)blocks), dim3(256), 0, stream, static_cast<const float*>(out),
                       static_cast<float*>(result), n, p.ksplit, (int64_t)p.split_stride);
  }
  return hipGetLastError() == hipSuccess ? SYNO_OK : SYNO_ERR_HIP;
}

namespace {
PhaseParams phase_params(const ConvLike& c, int s, int window) {
  PhaseParams q{};
  q.O = c.Og; q.C = c.Cg; q.K = c.KH; q.s = s; q.p = c.ph; q.window = window;
  q.ws_o = c.ws_o; q.ws_c = c.ws_c; q.ws_kh = c.ws_kh; q.ws_kw = c.ws_kw;
  return q;
}
}  // namespace

syno_status launch_phase_weight_gather(const ConvLike& c, int s, int window, const float* dWp, float* dW, hipStream_t stream) {
  const PhaseParams q = phase_params(c, s, window);
  const int64_t n = (int64_t)q.O * q.C * q.K * q.K;
  if (n >= (1ll << 31)) return SYNO_ERR_SHAPE;
  hipLaunchKernelGGL(phase_weight_gather, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, q, dWp, dW);
  return hipGetLastError() == hipSuccess ? SYNO_OK : SYNO_ERR_HIP;
}

syno_status launch_phase_weight_build(const ConvLike& c, int s, int window, int elem_bytes, const void* W, void* Wpp, hipStream_t stream) {
  const PhaseParams q = phase_params(c, s, window);
  const int64_t n = (int64_t)q.C * q.s * q.s * q.O * window * window;
  if (n >= (1ll << 31)) return SYNO_ERR_SHAPE;
  const dim3 grid((unsigned)((n + 255) / 256));
  if (elem_bytes == 4)
    hipLaunchKernelGGL(phase_weight_build<uint32_t>, grid, dim3(256), 0, stream, q, static_cast<const uint32_t*>(W), static_cast<uint32_t*>(Wpp));
  else
    hipLaunchKernelGGL(phase_weight_build<uint16_t>, grid, dim3(256), 0, stream, q, static_cast<const uint16_t*>(W), static_cast<uint16_t*>(Wpp));
  return hipGetLastError() == hipSuccess ? SYNO_OK : SYNO_ERR_HIP;
}

syno_status launch_transpose_2d(const void* src, void* dst, int64_t rows, int64_t cols, int elem_bytes, hipStream_t stream) {
  if (rows < 1 || cols < 1 || rows >= (1ll << 31) || cols >= (1ll << 31) || (rows + 31) / 32 > 65535) return SYNO_ERR_SHAPE;
  const dim3 grid((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32));
  if (elem_bytes == 4)
    hipLaunchKernelGGL(transpose_2d<uint32_t>, grid, dim3(256), 0, stream, static_cast<const uint32_t*>(src), static_cast<uint32_t*>(dst), (int)rows, (int)cols);
  else if (elem_bytes == 2)
    hipLaunchKernelGGL(transpose_2d<uint16_t>, grid, dim3(256), 0, stream, static_cast<const uint16_t*>(src), static_cast<uint16_t*>(dst), (int)rows, (int)cols);
  else
    return SYNO_ERR_UNSUPPORTED;
  return hipGetLastError() == hipSuccess ? SYNO_OK : SYNO_ERR_HIP;
}

}  // namespace syno
