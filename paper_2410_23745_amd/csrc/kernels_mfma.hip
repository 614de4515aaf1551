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
#include <string>
#include <type_traits>

#include "plan.h"

namespace syno {

struct MfmaParams {
  // problem, in forward terms
  int32_t G, Og, Cg, Ho, Wo, Hi, Wi, KH, KW, ph, pw;
  int32_t rows_total;                 // N*Ho output rows
  int32_t h_wrap, h_shift, h_shift_g; // cyclic rows: input row = (h + h_shift + h_shift_g*g) mod Hi  (KH = 1)
  int32_t xs_n, xs_c;                 // source strides: image, channel (rows are Wi apart, columns adjacent)
  int32_t os_n, os_o;                 // result strides: image, channel
  int32_t ws_g, ws_o, ws_c, ws_kh, ws_kw, w_base;
  // tiling
  int32_t TR, BN, KC, n_mblocks, n_nblocks, n_chunks;
  int32_t n_slots, Wp, cgrps;
  int32_t w_row;                      // LDS weight row pitch (elements)
  int32_t lds_w_off, lds_tab_off, lds_bytes;
  int32_t w_block;                    // bf16: elements of one packed weight block (KH*KW*BN*w_row)
  // ceil(2^32/d) for the divisors the kernel needs (exact quotients for n*d < 2^32, which the host checks)
  uint32_t m_wo, m_ho, m_wi, m_pcg, m_per_o, m_khw, m_kw;
};

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// n / d through the precomputed m = ceil(2^32/d) (m = 0 stands for d = 1, whose constant does not fit)
__device__ __forceinline__ int fdiv(int n, uint32_t m) { return m ? (int)__umulhi((uint32_t)n, m) : n; }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Source of each row slot: element offset of the input row inside the tensor, or -1 when the slot
// is padding (above/below the image, or beyond the rows this block owns).
__device__ __forceinline__ int slot_source(const MfmaParams& p, int R0, int rows, int g, int s) {
  if (p.h_wrap) {
    if (s >= rows) return -1;
    const int rho = R0 + s, n = rho / p.Ho, h = rho - n * p.Ho;
    const int r = (h + p.h_shift + p.h_shift_g * g) % p.Hi;
    return n * p.xs_n + r * p.Wi;
  }
  int rho = R0, s0 = 0;
  const int end = R0 + rows;
  while (rho < end) {
    const int n = rho / p.Ho, h = rho - n * p.Ho;
    const int seg_rows = min(p.Ho - h, end - rho);
    const int seg_slots = seg_rows + p.KH - 1;
    if (s < s0 + seg_slots) {
      const int r = h + (s - s0) - p.ph;
      return (r >= 0 && r < p.Hi) ? n * p.xs_n + r * p.Wi : -1;
    }
    s0 += seg_slots;
    rho += seg_rows;
  }
  return -1;
}

// First slot of output row i of the block (tap kh adds kh slots).
__device__ __forceinline__ int slot_of_row(const MfmaParams& p, int R0, int i) {
  if (p.h_wrap) return i;
  return i + (p.KH - 1) * (fdiv(R0 + i, p.m_ho) - fdiv(R0, p.m_ho));
}

// bf16 only: W[g][o][c][kh][kw] (any strides) -> blocks [g][nb][chunk] of [tap][o_local][w_row] with the
// channel innermost; rows beyond Og / Cg and the row padding are zero.  One thread gathers the 8
// channels of one 16-byte piece.
__global__ __launch_bounds__(256) void pack_weight_bf16(const MfmaParams p, const uint16_t* __restrict__ Wt,
                                                        uint4* __restrict__ packed, int64_t pieces) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= pieces) return;
  const int KHW = p.KH * p.KW, row8 = p.w_row >> 3;
  int64_t r = i;
  const int cq = (int)(r % row8); r /= row8;
  const int ol = (int)(r % p.BN); r /= p.BN;
  const int tap = (int)(r % KHW); r /= KHW;
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
  packed[i] = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
}

// BF = false: fp32 inputs, CI = 4, v_mfma_f32_16x16x4_f32  (A: lane -> row l%16, k = l/16).
// BF = true : bf16 inputs, CI = 8, v_mfma_f32_16x16x32_bf16 (A: lane -> row l%16, k = 8*(l/16)..+7);
//             `Wv` is the packed copy.
// WNAT (fp32 only): the weight block of one output channel, [KC][KH][KW], is contiguous and 16-byte
//             aligned in memory, so it is staged with 16-byte loads instead of element by element.
// WK:  waves that share one output tile and split each chunk's k-steps among themselves (for shapes whose
//      per-SIMD share of the output is only a few MFMA tiles: a wave then still issues TM*TN MFMAs per
//      LDS round trip); their accumulators are added through LDS at the end.
template <bool BF, bool WNAT, int WM, int WN, int WK, int TM, int TN, int XI, int WI, bool ONE, bool OUTBF>
__global__ __launch_bounds__(WM* WN* WK * 64) void conv_mfma(const MfmaParams p, const void* __restrict__ Xv,
                                                         const void* __restrict__ Wv, void* __restrict__ out) {
  constexpr int NT = WM * WN * WK * 64;
  constexpr int BN = WN * TN * 16;
  constexpr int CI = BF ? 8 : 4;
  constexpr int CG_STEP = BF ? 4 : 1;        // channel groups one MFMA consumes
  using XT = std::conditional_t<BF, uint16_t, float>;
  using Frag = std::conditional_t<BF, bf16x8, float>;
  constexpr bool W16 = BF || WNAT;           // weights move in 16-byte pieces
  using WReg = std::conditional_t<W16, uint4, float>;
  extern __shared__ __align__(16) unsigned char smem[];
  float4* xl = reinterpret_cast<float4*>(smem);
  int* slot_src = reinterpret_cast<int*>(smem + p.lds_tab_off);

  const int tid = threadIdx.x, lane = tid & 63;
  const int widx = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in an SGPR
  const int wk = widx / (WM * WN), wtile = widx - wk * (WM * WN);
  const int wn = wtile / WM;
  const int wm = (wtile + wn) % WM;         // spread the fuller wave rows over the SIMDs
  int bid = blockIdx.x;
  const int nb = bid % p.n_nblocks; bid /= p.n_nblocks;
  const int mb = bid % p.n_mblocks;
  const int g = bid / p.n_mblocks;
  const int R0 = mb * p.TR;
  const int rows = min(p.TR, p.rows_total - R0);
  const int KHW = p.KH * p.KW;

  for (int s = tid; s < p.n_slots; s += NT) slot_src[s] = slot_source(p, R0, rows, g, s);
  {
    const int n16 = p.cgrps * p.n_slots * p.Wp;
    for (int i = tid; i < n16; i += NT) xl[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  __syncthreads();

  // ---- loop-invariant descriptors of what this thread stages per chunk
  const XT* Xg = reinterpret_cast<const XT*>(Xv) + (int64_t)g * p.Cg * p.xs_c;
  int x_goff[XI], x_loff[XI], x_cg[XI];
  int w_goff[WI], w_meta[WI];   // fp32 meta: LDS dword offset | local channel << 20 | zero-fill << 29 | unused << 30
  const float* Wg32 = nullptr;
  const uint4* Wg16 = nullptr;
  {
    const int per_cg = p.n_slots * p.Wi, total = p.cgrps * per_cg;
#pragma unroll
    for (int k = 0; k < XI; ++k) {
      const int idx = tid + k * NT;
      const int cg = fdiv(idx, p.m_pcg), rem = idx - cg * per_cg;
      const int s = fdiv(rem, p.m_wi), x = rem - s * p.Wi;
      const int src = idx < total ? slot_src[s] : -1;
      x_goff[k] = src >= 0 ? src + x + cg * CI * p.xs_c : -1;
      x_loff[k] = (cg * p.n_slots + s) * p.Wp + x + p.pw;
      x_cg[k] = cg * CI;
    }
  }
  // fp32: one weight element per item, gathered with the operator's strides into [o][c*KHW+tap].
  // bf16: 16-byte pieces of this block's packed image, copied as they are.
  if constexpr (BF) {
    Wg16 = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(Wv) +
                                          ((int64_t)(g * p.n_nblocks + nb) * p.n_chunks) * p.w_block);
    const int units = p.w_block >> 3;
#pragma unroll
    for (int k = 0; k < WI; ++k) {
      const int idx = tid + k * NT;
      w_goff[k] = idx < units ? idx : -1;
      w_meta[k] = 0;
    }
  } else if constexpr (WNAT) {
    Wg32 = reinterpret_cast<const float*>(Wv) + (int64_t)g * p.ws_g + (int64_t)nb * BN * p.ws_o;
    const int per_o4 = (p.KC * KHW) >> 2, total = BN * per_o4;   // float4 pieces per output channel
#pragma unroll
    for (int k = 0; k < WI; ++k) {
      const int idx = tid + k * NT;
      const int o = fdiv(idx, p.m_per_o), e4 = idx - o * per_o4;
      const bool ok = idx < total && nb * BN + o < p.Og;
      w_goff[k] = ok ? o * p.ws_o + e4 * 4 : -1;                 // element offset
      w_meta[k] = idx < total ? (o * p.w_row + e4 * 4) >> 2 : -1; // LDS float4 index
    }
  } else {
    Wg32 = reinterpret_cast<const float*>(Wv) + p.w_base + (int64_t)g * p.ws_g + (int64_t)nb * BN * p.ws_o;
    const int per_o = p.KC * KHW, total = BN * per_o;
#pragma unroll
    for (int k = 0; k < WI; ++k) {
      const int idx = tid + k * NT;
      const int o = fdiv(idx, p.m_per_o), e = idx - o * per_o;
      const int cl = fdiv(e, p.m_khw), tap = e - cl * KHW;
      const int kh = fdiv(tap, p.m_kw), kw = tap - kh * p.KW;
      const bool ok = idx < total && nb * BN + o < p.Og;
      // tap strides may be negative (reversed taps of the adjoint), so validity lives in the meta word
      w_goff[k] = ok ? o * p.ws_o + cl * p.ws_c + kh * p.ws_kh + kw * p.ws_kw : 0;
      w_meta[k] = (idx < total ? o * p.w_row + e : 0) | (cl << 20) | (ok ? 0 : (1 << 29)) | (idx < total ? 0 : (1 << 30));
    }
  }
  // ---- per-lane operand bases; the block's MT row tiles are dealt out evenly to the wave rows
  const int block_px = rows * p.Wo;
  const int MT = (block_px + 15) >> 4;
  const int tiles_base = MT / WM, tiles_extra = MT - tiles_base * WM;
  const int my_tiles = tiles_base + (wm < tiles_extra ? 1 : 0);
  const int my_first = wm * tiles_base + min(wm, tiles_extra);
  const int cg_stride = p.n_slots * p.Wp;          // 16-byte units between channel groups
  int a_base[TM];                                   // fp32: dword index; bf16: 16-byte unit index
#pragma unroll
  for (int t = 0; t < TM; ++t) {
    int m = (my_first + t) * 16 + (lane & 15);
    if (t >= my_tiles || m >= block_px) m = 0;
    const int i = fdiv(m, p.m_wo), w = m - i * p.Wo;
    const int px = slot_of_row(p, R0, i) * p.Wp + w;
    a_base[t] = BF ? px + (lane >> 4) * cg_stride : px * 4 + (lane >> 4);
  }
  int b_base[TN];                                   // fp32: dword index; bf16: element index
#pragma unroll
  for (int u = 0; u < TN; ++u) {
    const int ol = (wn * TN + u) * 16 + (lane & 15);
    b_base[u] = BF ? ol * p.w_row + (lane >> 4) * 8 : ol * p.w_row + (lane >> 4) * KHW;
  }

  // Everything from here on is instantiated once per possible tile count of a wave, so that the
  // accumulators and fragments of a wave with fewer row tiles do not occupy registers and the MFMA
  // block is straight-line code.
  auto run = [&](auto ntl_c) {
  constexpr int NTL = decltype(ntl_c)::value;
  constexpr int NA = NTL > 0 ? NTL : 1;
  floatx4 acc[NA][TN];
#pragma unroll
  for (int t = 0; t < NA; ++t)
#pragma unroll
    for (int u = 0; u < TN; ++u) acc[t][u] = floatx4{0.f, 0.f, 0.f, 0.f};

  XT xr[XI][CI];
  WReg wr[WI];
  // Loads use a wave-uniform base plus 32-bit byte offsets.  Items without a source read offset 0 (any
  // valid address) and are simply not written to LDS, so the common path has no per-load predicate.
  const bool chan_tail = (p.Cg % p.KC) != 0;
  const char* xbase = reinterpret_cast<const char*>(Xg);
  auto fetch = [&](int ch) {
    const int c0 = ch * p.KC;
    if (!chan_tail) {
#pragma unroll
      for (int k = 0; k < XI; ++k) {
        const uint32_t o = (uint32_t)(max(x_goff[k], 0) + c0 * p.xs_c) * (uint32_t)sizeof(XT);
#pragma unroll
        for (int j = 0; j < CI; ++j)
          xr[k][j] = *reinterpret_cast<const XT*>(xbase + (o + (uint32_t)(j * p.xs_c) * (uint32_t)sizeof(XT)));
      }
    } else {
#pragma unroll
      for (int k = 0; k < XI; ++k)
#pragma unroll
        for (int j = 0; j < CI; ++j) {
          const int c = c0 + x_cg[k] + j;
          xr[k][j] = (x_goff[k] >= 0 && c < p.Cg) ? Xg[x_goff[k] + (int64_t)(c0 + j) * p.xs_c] : XT(0);
        }
    }
    if constexpr (BF) {
      const uint4* src = Wg16 + (int64_t)ch * (p.w_block >> 3);
#pragma unroll
      for (int k = 0; k < WI; ++k) wr[k] = w_goff[k] >= 0 ? src[w_goff[k]] : make_uint4(0, 0, 0, 0);
    } else if constexpr (WNAT) {
      // (the planner only picks this path when Cg is a multiple of KC, so no channel tail here)
#pragma unroll
      for (int k = 0; k < WI; ++k)
        wr[k] = w_goff[k] >= 0 ? *reinterpret_cast<const uint4*>(Wg32 + w_goff[k] + (int64_t)c0 * p.ws_c)
                               : make_uint4(0, 0, 0, 0);
    } else {
#pragma unroll
      for (int k = 0; k < WI; ++k) {
        const int cl = (w_meta[k] >> 20) & 511;
        wr[k] = (!(w_meta[k] >> 29) && c0 + cl < p.Cg) ? Wg32[w_goff[k] + (int64_t)c0 * p.ws_c] : 0.f;
      }
    }
  };
  auto stage = [&]() {
#pragma unroll
    for (int k = 0; k < XI; ++k)
      if (x_goff[k] >= 0) {
        if constexpr (BF) {
          uint4 v;
          v.x = xr[k][0] | ((uint32_t)xr[k][1] << 16);
          v.y = xr[k][2] | ((uint32_t)xr[k][3] << 16);
          v.z = xr[k][4] | ((uint32_t)xr[k][5] << 16);
          v.w = xr[k][6] | ((uint32_t)xr[k][7] << 16);
          reinterpret_cast<uint4*>(xl)[x_loff[k]] = v;
        } else {
          xl[x_loff[k]] = make_float4(xr[k][0], xr[k][1], xr[k][2], xr[k][3]);
        }
      }
    if constexpr (BF) {
      uint4* wl = reinterpret_cast<uint4*>(smem + p.lds_w_off);
#pragma unroll
      for (int k = 0; k < WI; ++k)
        if (w_goff[k] >= 0) wl[w_goff[k]] = wr[k];
    } else if constexpr (WNAT) {
      uint4* wl = reinterpret_cast<uint4*>(smem + p.lds_w_off);
#pragma unroll
      for (int k = 0; k < WI; ++k)
        if (w_meta[k] >= 0) wl[w_meta[k]] = wr[k];
    } else {
      float* wl = reinterpret_cast<float*>(smem + p.lds_w_off);
#pragma unroll
      for (int k = 0; k < WI; ++k)
        if (!(w_meta[k] >> 30)) wl[w_meta[k] & 0xfffff] = wr[k];
    }
  };

  // ONE: the whole reduction fits one chunk, so the staging registers are dead once it is in LDS
  const int n_chunks = ONE ? 1 : p.n_chunks;
  fetch(0);
  for (int ch = 0; ch < n_chunks; ++ch) {
    __syncthreads();   // everyone has finished reading the previous chunk
    stage();
    __syncthreads();
    if (ch + 1 < n_chunks) fetch(ch + 1);   // next chunk travels while this one is computed
    // One k-step = CI*CG_STEP channels at one tap.  Fragments of step i+1 are read from LDS while the
    // MFMAs of step i issue.  The tile count is a compile-time constant per case so that the MFMA
    // block is straight-line code.
    if constexpr (NTL > 0) {
      const int all_steps = (p.cgrps / CG_STEP) * KHW;
      const int first = wk * all_steps / WK, steps = (wk + 1) * all_steps / WK - first;
      if (steps > 0) {
      // running operand offsets of the current k-step (wave-uniform, advanced with scalar adds):
      // fp32: a in dwords, b in dwords; bf16: a in 16-byte units, b in elements
      int cg = first / KHW, kh = (first - cg * KHW) / p.KW, kw = first - cg * KHW - kh * p.KW;
      const int a_kw = BF ? 1 : 4, a_kh = (BF ? 1 : 4) * p.Wp, a_cg = (BF ? CG_STEP : 4) * cg_stride;
      const int b_kw = BF ? BN * p.w_row : 1, b_cg = BF ? CG_STEP * CI : CI * KHW;
      int a_off = cg * a_cg + kh * a_kh + kw * a_kw;
      int b_off = BF ? (kh * p.KW + kw) * b_kw + cg * b_cg : cg * b_cg + kh * p.KW + kw;
      Frag a0[NTL], b0[TN], a1[NTL], b1[TN];
      auto read = [&](Frag (&a)[NTL], Frag (&b)[TN]) {
        if constexpr (BF) {
          const uint4* xq = reinterpret_cast<const uint4*>(smem);
          const uint16_t* wq = reinterpret_cast<const uint16_t*>(smem + p.lds_w_off);
#pragma unroll
          for (int u = 0; u < TN; ++u)
            b[u] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(wq + b_base[u] + b_off));
#pragma unroll
          for (int t = 0; t < NTL; ++t) a[t] = __builtin_bit_cast(bf16x8, xq[a_base[t] + a_off]);
        } else {
          const float* xq = reinterpret_cast<const float*>(smem);
          const float* wq = reinterpret_cast<const float*>(smem + p.lds_w_off);
#pragma unroll
          for (int u = 0; u < TN; ++u) b[u] = wq[b_base[u] + b_off];
#pragma unroll
          for (int t = 0; t < NTL; ++t) a[t] = xq[a_base[t] + a_off];
        }
      };
      auto advance = [&]() {
        a_off += a_kw; b_off += b_kw;
        if (++kw == p.KW) {
          kw = 0; a_off += a_kh - p.KW * a_kw;
          if (++kh == p.KH) {
            kh = 0; a_off += a_cg - p.KH * a_kh;
            b_off += b_cg - KHW * b_kw;
          }
        }
      };
      auto mfmas = [&](const Frag (&a)[NTL], const Frag (&b)[TN]) {
#pragma unroll
        for (int t = 0; t < NTL; ++t)
#pragma unroll
          for (int u = 0; u < TN; ++u) {
            if constexpr (BF) acc[t][u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[t], b[u], acc[t][u], 0, 0, 0);
            else acc[t][u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[t], b[u], acc[t][u], 0, 0, 0);
          }
      };
      // steady state without branches, so that the waits on LDS can be exact: the reads of the next
      // step stay in flight while the MFMAs of the current one issue
      read(a0, b0);
      int it = 0;
      for (; it + 2 < steps; it += 2) {
        advance(); read(a1, b1); mfmas(a0, b0);
        advance(); read(a0, b0); mfmas(a1, b1);
      }
      if (it + 1 < steps) { advance(); read(a1, b1); mfmas(a0, b0); mfmas(a1, b1); }
      else mfmas(a0, b0);
      }
    }
  }

  // ---- waves that split the k-steps add their accumulators into the first one's
  if constexpr (WK > 1) {
    floatx4* red = reinterpret_cast<floatx4*>(smem);     // [WM*WN][TM*TN][64 lanes], reusing the staging area
    for (int k = 1; k < WK; ++k) {
      __syncthreads();
      if (wk == k) {
#pragma unroll
        for (int t = 0; t < NTL; ++t)
#pragma unroll
          for (int u = 0; u < TN; ++u) red[((wtile * TM + t) * TN + u) * 64 + lane] = acc[t][u];
      }
      __syncthreads();
      if (wk == 0) {
#pragma unroll
        for (int t = 0; t < NTL; ++t)
#pragma unroll
          for (int u = 0; u < TN; ++u) acc[t][u] += red[((wtile * TM + t) * TN + u) * 64 + lane];
      }
    }
    if (wk != 0) return;
  }

  // ---- store: lane holds 4 consecutive pixels (rows of D) of one channel (column of D)
  const int img_px = p.Ho * p.Wo;
#pragma unroll
  for (int t = 0; t < NTL; ++t) {
    const int m0 = (my_first + t) * 16 + 4 * (lane >> 4);
#pragma unroll
    for (int u = 0; u < TN; ++u) {
      const int o = nb * BN + (wn * TN + u) * 16 + (lane & 15);
      if (o >= p.Og || m0 >= block_px) continue;
      // pixel m0 of the block -> (image, pixel inside the image)
      const int i0 = fdiv(m0, p.m_wo), rho = R0 + i0;
      const int n = fdiv(rho, p.m_ho), px = (rho - n * p.Ho) * p.Wo + (m0 - i0 * p.Wo);
      const int64_t off = (int64_t)n * p.os_n + (int64_t)(g * p.Og + o) * p.os_o + px;
      const bool together = m0 + 3 < block_px && px + 3 < img_px;
      if constexpr (OUTBF) {
        uint16_t* op = reinterpret_cast<uint16_t*>(out);
        if (together && (off & 3) == 0) {
          uint2 v;
          v.x = f32_to_bf16_rne(acc[t][u][0]) | ((uint32_t)f32_to_bf16_rne(acc[t][u][1]) << 16);
          v.y = f32_to_bf16_rne(acc[t][u][2]) | ((uint32_t)f32_to_bf16_rne(acc[t][u][3]) << 16);
          *reinterpret_cast<uint2*>(op + off) = v;
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (m0 + j < block_px) {
              const int ij = fdiv(m0 + j, p.m_wo), rj = R0 + ij, nj = fdiv(rj, p.m_ho);
              op[(int64_t)nj * p.os_n + (int64_t)(g * p.Og + o) * p.os_o + (rj - nj * p.Ho) * p.Wo + (m0 + j - ij * p.Wo)] =
                  f32_to_bf16_rne(acc[t][u][j]);
            }
        }
      } else {
        float* op = reinterpret_cast<float*>(out);
        if (together && (off & 3) == 0) {
          *reinterpret_cast<float4*>(op + off) = make_float4(acc[t][u][0], acc[t][u][1], acc[t][u][2], acc[t][u][3]);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (m0 + j < block_px) {
              const int ij = fdiv(m0 + j, p.m_wo), rj = R0 + ij, nj = fdiv(rj, p.m_ho);
              op[(int64_t)nj * p.os_n + (int64_t)(g * p.Og + o) * p.os_o + (rj - nj * p.Ho) * p.Wo + (m0 + j - ij * p.Wo)] =
                  acc[t][u][j];
            }
        }
      }
    }
  }
  };
  static_assert(TM <= 8, "extend the dispatch below");
  switch (my_tiles) {
    case 0: run(std::integral_constant<int, 0>{}); break;
    case 1: run(std::integral_constant<int, 1>{}); break;
    case 2: if constexpr (TM >= 2) run(std::integral_constant<int, 2>{}); break;
    case 3: if constexpr (TM >= 3) run(std::integral_constant<int, 3>{}); break;
    case 4: if constexpr (TM >= 4) run(std::integral_constant<int, 4>{}); break;
    case 5: if constexpr (TM >= 5) run(std::integral_constant<int, 5>{}); break;
    case 6: if constexpr (TM >= 6) run(std::integral_constant<int, 6>{}); break;
    case 7: if constexpr (TM >= 7) run(std::integral_constant<int, 7>{}); break;
    case 8: if constexpr (TM >= 8) run(std::integral_constant<int, 8>{}); break;
    default: break;
  }
}

// ---------------------------------------------------------------------------------------------
// Host side: tile choice and launch
// ---------------------------------------------------------------------------------------------
struct Variant {
  int WM, WN, WK, TM, TN, XI, WI;
  int KC;        // channels per chunk (fp32 variants may fall back to smaller multiples)
  bool wnat;     // fp32: contiguous weight rows staged in 16-byte pieces
  bool one;      // only for reductions that fit a single chunk (nothing is prefetched during the MFMAs)
  constexpr int NT() const { return WM * WN * WK * 64; }
  constexpr int BN() const { return WN * TN * 16; }
  constexpr int MT() const { return WM * TM; }
};
// Tile variants, 8 waves each.  Row tiles x column tiles per wave, waves along M x N x K:
//   fp32 0-2: any weight strides, 8 channels per chunk (the backward-data adjoint runs here)
//   fp32 3-8: forward weight layout [o][c][kh][kw], 16 or 32 channels per chunk (what fits the registers)
//   bf16 0-5: packed weights, 32 channels per chunk
//   bf16 6:   packed weights, at most 64 channels per group, staged in one go
constexpr int kNumF32Variants = 9, kNumBf16Variants = 7;
constexpr Variant kF32Variants[kNumF32Variants] = {
    {4, 2, 1, 7, 2, 3, 9, 8, false}, {4, 2, 1, 7, 1, 3, 5, 8, false}, {8, 1, 1, 4, 1, 3, 3, 8, false},
    {4, 2, 1, 7, 2, 4, 5, 16, true}, {4, 1, 2, 7, 2, 4, 3, 16, true}, {2, 1, 4, 7, 2, 4, 3, 16, true},
    {1, 1, 8, 4, 4, 4, 5, 16, true}, {4, 2, 1, 7, 1, 8, 5, 32, true}, {8, 1, 1, 4, 1, 8, 3, 32, true}};
constexpr Variant kBf16Variants[kNumBf16Variants] = {
    {4, 2, 1, 7, 2, 4, 6, 32, false}, {4, 1, 2, 7, 2, 4, 3, 32, false}, {2, 1, 4, 7, 2, 4, 3, 32, false},
    {1, 1, 8, 4, 4, 4, 6, 32, false}, {4, 2, 1, 7, 1, 4, 3, 32, false}, {8, 1, 1, 4, 1, 4, 2, 32, false},
    {4, 2, 1, 7, 2, 8, 11, 64, false, true}};
constexpr int kNumCU = 256;
constexpr int kMaxLdsBytes = 160 * 1024;   // all of a CU's LDS

int num_variants(bool bf) { return bf ? kNumBf16Variants : kNumF32Variants; }
const Variant& variant_of(bool bf, int vi) { return bf ? kBf16Variants[vi] : kF32Variants[vi]; }

// most images a run of TR consecutive output rows can touch (blocks start at multiples of TR)
int images_spanned(int TR, int Ho) {
  if (Ho % TR == 0) return 1;
  if (TR % Ho == 0) return TR / Ho;
  return (TR + Ho - 2) / Ho + 1;
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

// Parameter record of contraction `which` (forward, or backward-data as its adjoint) for tile variant vi
// and TR output rows per block.  False when the combination does not fit the kernel's static limits.
bool fill_params(const syno_plan* plan, int which, int vi, int TR, MfmaParams& p) {
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
  const int plane = c.Hi * c.Wi;
  if (which == SYNO_FWD) {
    p.Og = c.Og; p.Cg = c.Cg; p.ph = c.ph; p.pw = c.pw;
    p.h_shift = c.h_shift; p.h_shift_g = c.h_shift_g;
    p.xs_c = plane; p.xs_n = c.G * c.Cg * plane;
    p.os_o = plane; p.os_n = c.G * c.Og * plane;
    p.ws_g = c.ws_g; p.ws_o = c.ws_o; p.ws_c = c.ws_c; p.ws_kh = c.ws_kh; p.ws_kw = c.ws_kw; p.w_base = 0;
  } else {
    // dX[n,g*Cg+c,y,x] = sum_{o,kh',kw'} G[n,g*Og+o, y+kh'-(KH-1-ph), x+kw'-(KW-1-pw)] * W[g,o,c,KH-1-kh',KW-1-kw']
    p.Og = c.Cg; p.Cg = c.Og; p.ph = c.KH - 1 - c.ph; p.pw = c.KW - 1 - c.pw;
    p.h_shift = (c.Hi - c.h_shift % c.Hi) % c.Hi; p.h_shift_g = (c.Hi - c.h_shift_g % c.Hi) % c.Hi;
    p.xs_c = plane; p.xs_n = c.G * c.Og * plane;
    p.os_o = plane; p.os_n = c.G * c.Cg * plane;
    p.ws_g = c.ws_g; p.ws_o = c.ws_c; p.ws_c = c.ws_o; p.ws_kh = -c.ws_kh; p.ws_kw = -c.ws_kw;
    p.w_base = (c.KH - 1) * c.ws_kh + (c.KW - 1) * c.ws_kw;
  }
  p.TR = TR;
  p.BN = v.BN();
  const int KHW = c.KH * c.KW;
  const int CI = bf ? 8 : 4;
  if (bf) {
    p.KC = v.KC;
    if (v.one && p.Cg > p.KC) return false;
    p.w_row = p.KC + 8;                          // elements; 80- and 144-byte rows keep B-fragment reads conflict free
    p.w_block = KHW * p.BN * p.w_row;
    if ((p.w_block >> 3) > v.WI * v.NT()) return false;
  } else if (v.wnat) {
    if (which != SYNO_FWD || c.ws_kw != 1 || c.ws_kh != c.KW || c.ws_c != KHW || (c.ws_o & 3) || (c.ws_g & 3))
      return false;
    p.KC = v.KC;
    while (p.KC > 8 && (p.Cg % p.KC != 0 || p.BN * p.KC * KHW > 4 * v.WI * v.NT() ||
                        (p.KC / CI) * (c.h_wrap ? TR : TR + (c.KH - 1) * images_spanned(TR, c.Ho)) * c.Wi > v.XI * v.NT()))
      p.KC -= 8;
    if (p.Cg % p.KC != 0 || ((p.KC * KHW) & 3) || p.BN * p.KC * KHW > 4 * v.WI * v.NT()) return false;
    p.w_row = pick_w_row(p.KC * KHW, KHW, 4);
  } else {
    p.KC = v.KC;
    while (p.KC > 4 && (p.BN * p.KC * KHW > v.WI * v.NT())) p.KC -= 4;
    if (p.BN * p.KC * KHW > v.WI * v.NT()) return false;
    p.w_row = pick_w_row(p.KC * KHW, KHW, 1);
  }
  p.cgrps = p.KC / CI;
  p.n_chunks = (p.Cg + p.KC - 1) / p.KC;
  p.n_mblocks = (p.rows_total + TR - 1) / TR;
  p.n_nblocks = (p.Og + p.BN - 1) / p.BN;
  p.n_slots = c.h_wrap ? TR : TR + (c.KH - 1) * images_spanned(TR, c.Ho);
  p.Wp = c.Wi + c.KW - 1;
  if ((TR * c.Wo + 15) / 16 > v.MT()) return false;
  if (p.cgrps * p.n_slots * c.Wi > v.XI * v.NT()) return false;
  const int x_bytes = p.cgrps * p.n_slots * p.Wp * 16;
  p.lds_w_off = x_bytes;
  const int w_bytes = bf ? p.w_block * 2 : p.BN * p.w_row * 4;
  p.lds_tab_off = p.lds_w_off + ((w_bytes + 15) & ~15);
  p.lds_bytes = p.lds_tab_off + ((p.n_slots * 4 + 15) & ~15);
  if (v.WK > 1) p.lds_bytes = std::max(p.lds_bytes, v.WM * v.WN * v.TM * v.TN * 1024);
  if (!bf && p.w_row * p.BN >= (1 << 20)) return false;
  auto magic = [](int64_t d) { return (uint32_t)(((1ull << 32) + d - 1) / std::max<int64_t>(d, 1)); };
  const int64_t per_cg = (int64_t)p.n_slots * c.Wi;
  const int64_t per_o = bf ? 1 : (v.wnat ? (p.KC * KHW) >> 2 : p.KC * KHW);
  // largest numerators: item indices (< XI*NT, WI*NT), pixels of a block (< 16*MT), output rows (< rows_total)
  const int64_t max_idx = (int64_t)std::max(v.XI, v.WI) * v.NT();
  if (max_idx * per_cg >= (1ll << 32) || max_idx * per_o >= (1ll << 32) || (int64_t)p.rows_total * c.Ho >= (1ll << 32))
    return false;
  p.m_wo = magic(c.Wo); p.m_ho = magic(c.Ho); p.m_wi = magic(c.Wi); p.m_pcg = magic(per_cg);
  p.m_per_o = magic(per_o); p.m_khw = magic(KHW); p.m_kw = magic(c.KW);
  return p.lds_bytes <= kMaxLdsBytes;
}

// Estimated duration of the launch in SIMD cycles.  Row tiles are dealt evenly to the WM wave rows, wave
// widx runs on SIMD widx%4, a 16x16 MFMA occupies its SIMD's matrix pipe for 32 (fp32 K=4) or 16 (bf16
// K=32) cycles, and one k-step of a wave cannot finish faster than its LDS reads allow.  Staging, barriers
// and the prologue overlap with another resident workgroup's MFMAs only when more than one fits on a CU.
double tile_cost(const MfmaParams& p, const Variant& v, const ConvLike& c, bool bf) {
  const int64_t wgs = (int64_t)p.n_mblocks * p.n_nblocks * c.G;
  const int MT = (std::min(p.TR, p.rows_total) * c.Wo + 15) / 16;
  const int base = MT / v.WM, extra = MT % v.WM;
  const double mfma_cycles = bf ? 16.0 : 32.0, read_cycles = bf ? 16.0 : 8.0;
  // per k-step of the chunk: cycles of matrix pipe and of step latency each SIMD sees, averaged over the
  // waves that split the steps
  double simd_mfma[4] = {0, 0, 0, 0}, simd_lat[4] = {0, 0, 0, 0};
  for (int widx = 0; widx < v.WM * v.WN * v.WK; ++widx) {
    const int wtile = widx % (v.WM * v.WN);
    const int wn = wtile / v.WM, wm = (wtile + wn) % v.WM;
    const int tiles = base + (wm < extra ? 1 : 0);
    if (!tiles) continue;
    simd_mfma[widx & 3] += mfma_cycles * tiles * v.TN / v.WK;
    // a wave's step: address arithmetic, LDS round trip, then its MFMAs issue
    simd_lat[widx & 3] += (200.0 + read_cycles * (tiles + v.TN)) / v.WK;
  }
  double step = 0;
  for (int s = 0; s < 4; ++s) step = std::max(step, std::max(simd_mfma[s], 0.5 * simd_lat[s] + 0.5 * simd_mfma[s]));
  const double steps = (double)p.n_chunks * (p.cgrps / (bf ? 4 : 1)) * c.KH * c.KW;
  const double overhead = p.n_chunks * 2500.0 + 6000.0 + (v.WK - 1) * 1500.0;
  const int resident = 1;   // 8 waves of up to 256 VGPRs fill a CU's register file
  const double per_cu_wgs = std::ceil((double)wgs / kNumCU);
  return per_cu_wgs * steps * step + std::ceil(per_cu_wgs / resident) * overhead;
}

template <bool BF, int VI, bool OUTBF>
void launch_variant(const MfmaParams& p, const void* X, const void* W, void* out, hipStream_t s) {
  constexpr Variant v = BF ? kBf16Variants[VI % kNumBf16Variants] : kF32Variants[VI];
  const int grid = p.n_mblocks * p.n_nblocks * p.G;
  auto kernel = conv_mfma<BF, v.wnat, v.WM, v.WN, v.WK, v.TM, v.TN, v.XI, v.WI, v.one, OUTBF>;
  static const hipError_t lds_opt_in =      // once per instantiation: allow more than the default 64 KB
      hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
  (void)lds_opt_in;
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(v.NT()), p.lds_bytes, s, p, X, W, out);
}

template <bool BF, bool OUTBF>
void launch_dtype(int vi, const MfmaParams& p, const void* X, const void* W, void* out, hipStream_t s) {
  switch (vi) {
    case 0: launch_variant<BF, 0, OUTBF>(p, X, W, out, s); break;
    case 1: launch_variant<BF, 1, OUTBF>(p, X, W, out, s); break;
    case 2: launch_variant<BF, 2, OUTBF>(p, X, W, out, s); break;
    case 3: launch_variant<BF, 3, OUTBF>(p, X, W, out, s); break;
    case 4: launch_variant<BF, 4, OUTBF>(p, X, W, out, s); break;
    case 5: launch_variant<BF, 5, OUTBF>(p, X, W, out, s); break;
    case 6: launch_variant<BF, 6, OUTBF>(p, X, W, out, s); break;
    case 7: if constexpr (!BF) launch_variant<BF, 7, OUTBF>(p, X, W, out, s); break;
    case 8: if constexpr (!BF) launch_variant<BF, 8, OUTBF>(p, X, W, out, s); break;
    default: break;
  }
}

size_t packed_weight_bytes(const MfmaParams& p) {
  return (size_t)p.G * p.n_nblocks * p.n_chunks * p.w_block * 2;
}

}  // namespace

bool mfma_supports(const syno_plan* p, int which) {
  if (!p->conv_like || which == SYNO_BWD_WEIGHT) return false;
  if (p->in_dtype == SYNO_F32 && p->out_dtype != SYNO_F32) return false;   // not instantiated
  const ConvLike& c = p->conv;
  if (c.sh != 1 || c.sw != 1 || c.w_wrap) return false;
  if (c.h_wrap && c.KH != 1) return false;
  if (c.Wi != c.Wo || c.Hi != c.Ho) return false;
  if (c.ph >= c.KH || c.pw >= c.KW) return false;
  if (c.Og == 1 && c.Cg == 1) return false;          // no contraction to speak of
  MfmaParams mp;
  for (int vi = 0; vi < num_variants(p->in_dtype == SYNO_BF16); ++vi)
    for (int TR = 1; TR <= c.N * c.Ho && TR * c.Wo <= 16 * 32; ++TR)
      if (fill_params(p, which, vi, TR, mp)) return true;
  return false;
}

void mfma_configure(syno_plan* plan, int which) {
  const ConvLike& c = plan->conv;
  const bool bf = plan->in_dtype == SYNO_BF16;
  double best = 1e300;
  int best_v = -1, best_tr = 0;
  MfmaParams mp;
  // SYNO_MFMA_TILE="variant,rows" overrides the tile choice (tuning aid)
  if (const char* f = getenv("SYNO_MFMA_TILE")) {
    int vi = -1, tr = 0;
    if (sscanf(f, "%d,%d", &vi, &tr) == 2 && fill_params(plan, which, vi, tr, mp)) {
      best_v = vi; best_tr = tr;
    }
  }
  if (best_v < 0)
    for (int vi = 0; vi < num_variants(bf); ++vi)
      for (int TR = 1; TR <= c.N * c.Ho && TR * c.Wo <= 16 * 32; ++TR) {
        if (!fill_params(plan, which, vi, TR, mp)) continue;
        const double cost = tile_cost(mp, variant_of(bf, vi), c, bf);
        if (cost < best) { best = cost; best_v = vi; best_tr = TR; }
      }
  fill_params(plan, which, best_v, best_tr, mp);
  plan->launch[which].variant = best_v * 4096 + best_tr;
  plan->launch[which].workspace = bf ? packed_weight_bytes(mp) : 0;
}

std::string mfma_describe(const syno_plan* plan, int which) {
  const int vi = plan->launch[which].variant / 4096, TR = plan->launch[which].variant % 4096;
  MfmaParams p;
  if (!fill_params(plan, which, vi, TR, p)) return "unconfigured";
  const Variant& v = variant_of(plan->in_dtype == SYNO_BF16, vi);
  char b[256];
  snprintf(b, sizeof b, "variant=%d rows/block=%d BN=%d KC=%d waves=%dx%dx%d grid=%d lds=%dB slots=%d", vi, TR, v.BN(),
           p.KC, v.WM, v.WN, v.WK, p.n_mblocks * p.n_nblocks * p.G, p.lds_bytes, p.n_slots);
  return b;
}

syno_status launch_mfma(const syno_plan* plan, int which, const void* A, const void* B, void* out, void* ws,
                        hipStream_t stream) {
  const int vi = plan->launch[which].variant / 4096, TR = plan->launch[which].variant % 4096;
  MfmaParams p;
  if (!fill_params(plan, which, vi, TR, p)) return SYNO_ERR_UNSUPPORTED;
  const bool obf = plan->out_dtype == SYNO_BF16;
  if (plan->in_dtype == SYNO_BF16) {
    if (!ws) return SYNO_ERR_WORKSPACE;
    const int64_t pieces = (int64_t)packed_weight_bytes(p) / 16;
    hipLaunchKernelGGL(pack_weight_bf16, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, stream, p,
                       static_cast<const uint16_t*>(B), static_cast<uint4*>(ws), pieces);
    if (obf) launch_dtype<true, true>(vi, p, A, ws, out, stream);
    else launch_dtype<true, false>(vi, p, A, ws, out, stream);
  } else {
    if (obf) return SYNO_ERR_UNSUPPORTED;
    launch_dtype<false, false>(vi, p, A, B, out, stream);
  }
  return hipGetLastError() == hipSuccess ? SYNO_OK : SYNO_ERR_HIP;
}

}  // namespace syno
