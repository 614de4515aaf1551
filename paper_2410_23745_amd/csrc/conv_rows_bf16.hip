// MFMA contraction family, bf16 inputs, operators whose whole reduction fits LDS at once (at most 64 channels per
// group): the grouped shift-unfold operator, the 64-channel convolution, their backward-data adjoints.
//   out[n, g*Og+o, h, w] = sum_{c,kh,kw} X[n, g*Cg+c, row(h,kh,g), w+kw-pw] * W[g,o,c,kh,kw]
// These shapes sit below the bf16 ridge point: the bytes bound them, not the matrix cores, and a launch lasts a few
// microseconds.  So the kernel is built to keep memory requests in flight rather than around the MFMA loop:
//   - small workgroups (4 waves) with little enough LDS that two or three share a compute unit and drift apart;
//   - a workgroup stages its 64 x Cg x taps weight block ONCE and then walks over row tiles of one (group, channel
//     block) pair; the input rows of the next tile are requested before the current tile is multiplied and their
//     LDS copy is double-buffered, so a tile costs one barrier and its loads, MFMAs and stores overlap those of its
//     neighbours;
//   - results leave the accumulators as 16-byte stores that are never waited for.
// A tile is TR output rows of ONE image (tiles do not cross images), every input row it touches in an LDS slot of
// W + KW - 1 pixels whose edge pixels stay zero (Unfold's padding; rows outside the image are written as zeros), 8
// channels = 16 bytes per pixel, so that an MFMA operand fragment is one 16-byte LDS read and a window tap a constant
// offset.  Shift's cyclic row offset only changes which input row fills a slot.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <string>
#include <type_traits>

#include "plan.h"

namespace syno {

struct RowsParams {
  int32_t G, Og, Cg, Ho, Wo, Hi, Wi, ph, pw, N;
  int32_t h_wrap, h_shift, h_shift_g;   // cyclic rows: input row = (h + h_shift + h_shift_g*g) mod Hi  (KH = 1)
  int32_t xs_n, xs_c, os_n, os_o;       // source and result strides: image, channel
  int32_t w_mode;                       // 0: packed copy; 1: W[g][o][c][taps] as it lies; 2: the same, for the adjoint
  int32_t ws_g, ws_o, ws_c;             // (modes 1, 2) element strides of W: group, forward output channel, input channel
  int32_t TR, tpi, n_tiles;             // output rows per tile, tiles per image, N*tpi
  int32_t n_nblocks, S;                 // 64-channel blocks per group; workgroups per (group, block) pair
  int32_t n_slots, Wp, vpr, x_items;    // row slots per tile, slot pitch (pixels), staging items per row, items per tile
  int32_t cg_stride;                    // 16-byte units between channel octets: n_slots*Wp
  int32_t lds_xbuf, n_xbuf, lds_w_off, lds_bytes;
  int32_t out_bf16;
  uint32_t m_wo, m_vpr, m_pcg, m_tpi;   // ceil(2^32/d) for Wo, vpr, n_slots*vpr, tpi (0 stands for d = 1)
};

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t bf16x4_unaligned __attribute__((ext_vector_type(4), aligned(2)));
typedef uint32_t u32x4_unaligned __attribute__((ext_vector_type(4), aligned(2)));

constexpr int kWaves = 4, kThreads = kWaves * 64;
constexpr int kBN = 64;            // output channels per workgroup
constexpr int kKC = 64;            // channels per group held in LDS (groups with fewer are padded with zeros)
constexpr int kWRow = kKC + 8;     // LDS weight row pitch (elements): 144-byte rows keep fragment reads conflict free
constexpr int kMaxTM = 4;          // row tiles of 16 pixels per wave
constexpr int kMaxXI = 3;          // staging items (4 pixels x 8 channels) per thread and tile

__device__ __forceinline__ int fdiv(int n, uint32_t m) { return m ? (int)__umulhi((uint32_t)n, m) : n; }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Any weight layout -> [g][nb][tap][o_local (64)][kWRow], channel innermost, zeros beyond Og / Cg and in the row
// padding.  One thread gathers the 8 channels of one 16-byte piece.  (ws_kh / ws_kw may be negative: reversed taps
// of the adjoint, then w_base points at the last tap.)
__global__ __launch_bounds__(256) void rows_pack_weight(const uint16_t* __restrict__ Wt, uint4* __restrict__ packed,
                                                        int64_t pieces, int G, int n_nblocks, int T, int KW, int Og,
                                                        int Cg, int64_t w_base, int ws_g, int ws_o, int ws_c, int ws_kh,
                                                        int ws_kw) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= pieces) return;
  constexpr int row8 = kWRow / 8;
  int64_t r = i;
  const int cq = (int)(r % row8); r /= row8;
  const int ol = (int)(r % kBN); r /= kBN;
  const int tap = (int)(r % T); r /= T;
  const int nb = (int)(r % n_nblocks);
  const int g = (int)(r / n_nblocks);
  const int o = nb * kBN + ol, c0 = cq * 8;
  const int kh = tap / KW, kw = tap - kh * KW;
  uint32_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    v[e] = 0;
    if (c0 + e < kKC && o < Og && c0 + e < Cg)
      v[e] = Wt[w_base + (int64_t)g * ws_g + (int64_t)o * ws_o + (int64_t)(c0 + e) * ws_c + kh * ws_kh + kw * ws_kw];
  }
  packed[i] = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
}

template <int KH, int KW>
__global__ __launch_bounds__(kThreads, 2) void conv_rows_bf16(const RowsParams p, const uint16_t* __restrict__ X,
                                                           const uint16_t* __restrict__ Wv, void* __restrict__ out) {
  constexpr int T = KH * KW;
  constexpr int KS = T * (kKC / 32);            // MFMA k-steps per tile: 32 channels at one tap each
  constexpr int B_TAP = kBN * kWRow * 2;        // bytes between taps of the weight block
  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  int bid = blockIdx.x;
  const int s_id = bid % p.S; bid /= p.S;
  const int nb = bid % p.n_nblocks;
  const int g = bid / p.n_nblocks;

  // ---- what this thread stages per tile: items of 4 adjacent pixels of one input row x 8 channels
  int x_slot[kMaxXI], x_col[kMaxXI], x_lds[kMaxXI], x_chan[kMaxXI];
#pragma unroll
  for (int k = 0; k < kMaxXI; ++k) {
    const int idx = tid + k * kThreads;
    const int cg = fdiv(idx, p.m_pcg), rem = idx - cg * (p.n_slots * p.vpr);
    const int s = fdiv(rem, p.m_vpr), x = min((rem - s * p.vpr) * 4, p.Wi - 4);   // a row's last item ends with the row
    x_slot[k] = idx < p.x_items ? s : -1;
    x_col[k] = x;
    x_chan[k] = cg * 8;
    x_lds[k] = (cg * p.n_slots + s) * p.Wp + x + p.pw;                             // 16-byte units
  }
  const uint16_t* Xg = X + (int64_t)g * p.Cg * p.xs_c;
  const bool chan_tail = (p.Cg & 7) != 0 || p.Cg < kKC;       // some of the 64 staged channels may not exist

  uint2 xr[kMaxXI][8];
  uint32_t x_ok = 0;       // bit k: item k of the tile in flight has a source row; bits 8.. : per item, channels that exist
  // requests the input rows of tile mb (all loads unconditional: what has no source reads the tensor's first
  // elements and is zeroed on its way into LDS)
  auto fetch = [&](int mb) {
    const int n = fdiv(mb, p.m_tpi), h0 = (mb - n * p.tpi) * p.TR;
    const int rows = min(p.TR, p.Ho - h0);
    x_ok = 0;
#pragma unroll
    for (int k = 0; k < kMaxXI; ++k) {
      const int s = x_slot[k];
      int r;
      bool ok;
      if (p.h_wrap) {
        r = (h0 + s + p.h_shift + p.h_shift_g * g) % p.Hi;
        ok = s >= 0 && s < rows;
      } else {
        r = h0 - p.ph + s;
        ok = s >= 0 && s < rows + KH - 1 && r >= 0 && r < p.Hi;
      }
      x_ok |= ok ? (1u << k) : 0u;
      const int base = ok ? n * p.xs_n + r * p.Wi + x_col[k] + x_chan[k] * p.xs_c : 0;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const bool cok = !chan_tail || x_chan[k] + j < p.Cg;
        const bf16x4_unaligned v = *reinterpret_cast<const bf16x4_unaligned*>(Xg + (ok && cok ? base + j * p.xs_c : 0));
        xr[k][j] = __builtin_bit_cast(uint2, v);
      }
    }
  };
  // registers -> LDS buffer `buf`: a pixel's 8 channels leave together as one 16-byte write
  auto stage = [&](int buf) {
    uint4* xl = reinterpret_cast<uint4*>(smem + buf * p.lds_xbuf);
#pragma unroll
    for (int k = 0; k < kMaxXI; ++k) {
      if (x_slot[k] < 0) continue;
      const bool ok = (x_ok >> k) & 1;
      uint32_t live[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) live[j] = (ok && (!chan_tail || x_chan[k] + j < p.Cg)) ? 0xffffffffu : 0u;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;     // high or low halves of (second, first)
        auto w = [&](int j) { return ((i >> 1) ? xr[k][j].y : xr[k][j].x) & live[j]; };
        uint4 v;
        v.x = __builtin_amdgcn_perm(w(1), w(0), sel);
        v.y = __builtin_amdgcn_perm(w(3), w(2), sel);
        v.z = __builtin_amdgcn_perm(w(5), w(4), sel);
        v.w = __builtin_amdgcn_perm(w(7), w(6), sel);
        xl[x_lds[k] + i] = v;
      }
    }
  };

  int mb = s_id;
  if (mb < p.n_tiles) fetch(mb);
  // while the first requests travel: zero both input buffers once (slot edges are the window's zero padding and are
  // never written afterwards), then bring the weight block in
  {
    uint4* z = reinterpret_cast<uint4*>(smem);
    const int n16 = (p.n_xbuf * p.lds_xbuf) >> 4;
    for (int i = tid; i < n16; i += kThreads) z[i] = make_uint4(0, 0, 0, 0);
  }
  if (p.w_mode == 0) {
    const uint4* src = reinterpret_cast<const uint4*>(Wv) + (int64_t)(g * p.n_nblocks + nb) * (T * kBN * kWRow / 8);
    uint4* wl = reinterpret_cast<uint4*>(smem + p.lds_w_off);
    for (int i = tid; i < T * kBN * kWRow / 8; i += kThreads) wl[i] = src[i];
  } else if (p.w_mode == 1) {
    // W[g][o][c][T taps]: a thread takes 8 channels x T taps of one output channel (T adjacent 16-byte loads) and
    // re-orders them into one 16-byte piece per tap
    const uint16_t* Wn = Wv + (int64_t)g * p.ws_g + (int64_t)nb * kBN * p.ws_o;
    uint4* wl = reinterpret_cast<uint4*>(smem + p.lds_w_off);
    for (int i = tid; i < kBN * (kKC / 8); i += kThreads) {
      const int octet = i % (kKC / 8), ol = i / (kKC / 8);
      const bool live = nb * kBN + ol < p.Og && octet * 8 < p.Cg;
      uint32_t in[4 * T];
#pragma unroll
      for (int q = 0; q < T; ++q) {
        u32x4_unaligned v = {0, 0, 0, 0};
        if (live) v = *reinterpret_cast<const u32x4_unaligned*>(Wn + (int64_t)ol * p.ws_o + octet * 8 * T + q * 8);
        in[4 * q + 0] = v[0]; in[4 * q + 1] = v[1]; in[4 * q + 2] = v[2]; in[4 * q + 3] = v[3];
      }
#pragma unroll
      for (int tap = 0; tap < T; ++tap) {
        uint32_t d[4];
#pragma unroll
        for (int h = 0; h < 4; ++h) {
          const int e0 = (2 * h) * T + tap, e1 = (2 * h + 1) * T + tap;
          const uint32_t sel = ((e0 & 1) ? 0x0302u : 0x0100u) | ((e1 & 1) ? 0x07060000u : 0x05040000u);
          d[h] = __builtin_amdgcn_perm(in[e1 >> 1], in[e0 >> 1], sel);
        }
        wl[(tap * kBN + ol) * (kWRow / 8) + octet] = make_uint4(d[0], d[1], d[2], d[3]);
      }
    }
  } else {
    // the adjoint's B operand out of the same memory: its rows are the forward input channels, its reduction runs
    // over the forward output channels, taps reversed: element (o, c, tap) goes to [T-1-tap][c][o].  (Here p.Og
    // counts forward input channels and p.Cg forward output channels.)
    const uint16_t* Wn = Wv + (int64_t)g * p.ws_g + (int64_t)nb * kBN * p.ws_c;
    uint16_t* wl = reinterpret_cast<uint16_t*>(smem + p.lds_w_off);
    // rows beyond the forward output channels and the row padding are never read; channels beyond Og read zeros
    for (int i = tid; i < kKC * (kBN / 8); i += kThreads) {
      const int octet = i % (kBN / 8), o = i / (kBN / 8);
      const bool live = o < p.Cg && nb * kBN + octet * 8 < p.Og;
      uint32_t in[4 * T];
#pragma unroll
      for (int q = 0; q < T; ++q) {
        u32x4_unaligned v = {0, 0, 0, 0};
        if (live) v = *reinterpret_cast<const u32x4_unaligned*>(Wn + (int64_t)o * p.ws_o + octet * 8 * T + q * 8);
        in[4 * q + 0] = v[0]; in[4 * q + 1] = v[1]; in[4 * q + 2] = v[2]; in[4 * q + 3] = v[3];
      }
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int tap = 0; tap < T; ++tap) {
          const int e = j * T + tap;
          wl[((T - 1 - tap) * kBN + octet * 8 + j) * kWRow + o] = (uint16_t)((e & 1) ? in[e >> 1] >> 16 : in[e >> 1]);
        }
    }
  }

  __syncthreads();     // the zero fill is complete before any input row is staged over it

  // ---- per-lane operand bases (the same for every tile): row tile t of this wave is tile wv + t*kWaves of the block
  int a_base[kMaxTM];
#pragma unroll
  for (int t = 0; t < kMaxTM; ++t) {
    int m = (wv + t * kWaves) * 16 + (lane & 15);
    if (m >= p.TR * p.Wo) m = 0;
    const int i = fdiv(m, p.m_wo), w = m - i * p.Wo;
    a_base[t] = (i * p.Wp + w + (lane >> 4) * p.cg_stride) * 16;
  }
  int b_base[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) b_base[u] = p.lds_w_off + ((u * 16 + (lane & 15)) * kWRow + (lane >> 4) * 8) * 2;
  // LDS byte offset of the A operand at k-step ks = (tap, 32-channel half)
  int a_step[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const int tap = ks / (kKC / 32), half = ks % (kKC / 32);
    a_step[ks] = ((tap / KW) * p.Wp + (tap % KW) + half * 4 * p.cg_stride) * 16;
  }

  int buf = 0;
  for (; mb < p.n_tiles; mb += p.S) {
    const int n = fdiv(mb, p.m_tpi), h0 = (mb - n * p.tpi) * p.TR;
    const int rows = min(p.TR, p.Ho - h0);
    const int block_px = rows * p.Wo;
    stage(buf);
    __syncthreads();     // this tile's rows (and, first time, the weights and the zero fill) are in LDS; every wave
                         // has left the tile before, whose buffer the tile after this one will overwrite
    if (mb + p.S < p.n_tiles) fetch(mb + p.S);
    const int MT = (block_px + 15) >> 4;
    const int my_tiles = wv < MT ? (MT - wv + kWaves - 1) / kWaves : 0;
    const int xoff = buf * p.lds_xbuf;

    auto run = [&](auto ntl_c) {
      constexpr int NTL = decltype(ntl_c)::value;
      floatx4 acc[NTL][4];
#pragma unroll
      for (int t = 0; t < NTL; ++t)
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[t][u] = floatx4{0.f, 0.f, 0.f, 0.f};
      uint4 fa[2][NTL], fb[2][4];
      auto read = [&](auto ks_c, uint4 (&a)[NTL], uint4 (&b)[4]) {
        constexpr int ks = decltype(ks_c)::value;
        constexpr int tap = ks / (kKC / 32), half = ks % (kKC / 32);
#pragma unroll
        for (int u = 0; u < 4; ++u) b[u] = *reinterpret_cast<const uint4*>(smem + b_base[u] + tap * B_TAP + half * 64);
#pragma unroll
        for (int t = 0; t < NTL; ++t) a[t] = *reinterpret_cast<const uint4*>(smem + xoff + a_base[t] + a_step[ks]);
      };
      auto step = [&](auto ks_c) {
        constexpr int ks = decltype(ks_c)::value;
        if constexpr (ks + 1 < KS) read(std::integral_constant<int, (ks + 1 < KS ? ks + 1 : 0)>{}, fa[(ks + 1) & 1], fb[(ks + 1) & 1]);
#pragma unroll
        for (int t = 0; t < NTL; ++t)
#pragma unroll
          for (int u = 0; u < 4; ++u)
            acc[t][u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fa[ks & 1][t]),
                                                                __builtin_bit_cast(bf16x8, fb[ks & 1][u]), acc[t][u], 0, 0, 0);
      };
      read(std::integral_constant<int, 0>{}, fa[0], fb[0]);
      auto steps = [&](auto self, auto ks_c) -> void {      // k-steps 0 .. KS-1, unrolled at compile time
        constexpr int ks = decltype(ks_c)::value;
        step(ks_c);
        if constexpr (ks + 1 < KS) self(self, std::integral_constant<int, ks + 1>{});
      };
      steps(steps, std::integral_constant<int, 0>{});

      // ---- store: a lane holds 4 consecutive pixels of one channel
      const int64_t img = (int64_t)n * p.os_n + (int64_t)h0 * p.Wo;
#pragma unroll
      for (int t = 0; t < NTL; ++t) {
        const int m0 = (wv + t * kWaves) * 16 + 4 * (lane >> 4);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int o = nb * kBN + u * 16 + (lane & 15);
          if (o >= p.Og || m0 >= block_px) continue;
          const int64_t off = img + (int64_t)(g * p.Og + o) * p.os_o + m0;
          const bool together = m0 + 3 < block_px && (off & 3) == 0;
          if (p.out_bf16) {
            uint16_t* op = reinterpret_cast<uint16_t*>(out) + off;
            if (together) {
              uint2 v;
              v.x = f32_to_bf16_rne(acc[t][u][0]) | ((uint32_t)f32_to_bf16_rne(acc[t][u][1]) << 16);
              v.y = f32_to_bf16_rne(acc[t][u][2]) | ((uint32_t)f32_to_bf16_rne(acc[t][u][3]) << 16);
              *reinterpret_cast<uint2*>(op) = v;
            } else {
#pragma unroll
              for (int j = 0; j < 4; ++j)
                if (m0 + j < block_px) op[j] = f32_to_bf16_rne(acc[t][u][j]);
            }
          } else {
            float* op = reinterpret_cast<float*>(out) + off;
            if (together) {
              *reinterpret_cast<float4*>(op) = make_float4(acc[t][u][0], acc[t][u][1], acc[t][u][2], acc[t][u][3]);
            } else {
#pragma unroll
              for (int j = 0; j < 4; ++j)
                if (m0 + j < block_px) op[j] = acc[t][u][j];
            }
          }
        }
      }
    };
    static_assert(kMaxTM == 4, "extend the dispatch below");
    switch (my_tiles) {
      case 1: run(std::integral_constant<int, 1>{}); break;
      case 2: run(std::integral_constant<int, 2>{}); break;
      case 3: run(std::integral_constant<int, 3>{}); break;
      case 4: run(std::integral_constant<int, 4>{}); break;
      default: break;
    }
    if (p.n_xbuf == 2) buf ^= 1;
    else __syncthreads();     // single buffer: everyone must have finished reading before the next tile is staged
  }
}

uint32_t magic_of(int64_t d) { return d < 2 ? 0u : (uint32_t)(((1ull << 32) + d - 1) / d); }

constexpr int kLdsLimit = 160 * 1024;

// Parameter record for contraction `which` with TR output rows per tile; false when the operator or the tile does
// not fit the kernel.
bool rows_fill(const syno_plan* plan, int which, int TR, RowsParams& p) {
  const ConvLike& c = plan->conv;
  p = RowsParams{};
  if (plan->in_dtype != SYNO_BF16 || which == SYNO_BWD_WEIGHT) return false;
  if (c.sh != 1 || c.sw != 1 || c.w_wrap || (c.h_wrap && c.KH != 1)) return false;
  if (c.Wi != c.Wo || c.Hi != c.Ho || c.ph >= c.KH || c.pw >= c.KW) return false;
  if (!((c.KH == 1 || c.KH == 3) && (c.KW == 1 || c.KW == 3))) return false;
  if (c.Wi < 4 || TR < 1 || TR > c.Ho) return false;
  const bool fwd = which == SYNO_FWD;
  p.G = c.G; p.Ho = c.Ho; p.Wo = c.Wo; p.Hi = c.Hi; p.Wi = c.Wi; p.N = c.N;
  p.Og = fwd ? c.Og : c.Cg; p.Cg = fwd ? c.Cg : c.Og;
  if (p.Cg > kKC || (p.Og == 1 && p.Cg == 1)) return false;
  p.ph = fwd ? c.ph : c.KH - 1 - c.ph; p.pw = fwd ? c.pw : c.KW - 1 - c.pw;
  p.h_wrap = c.h_wrap;
  p.h_shift = fwd ? c.h_shift : (c.Hi - c.h_shift % c.Hi) % c.Hi;
  p.h_shift_g = fwd ? c.h_shift_g : (c.Hi - c.h_shift_g % c.Hi) % c.Hi;
  const int plane = c.Hi * c.Wi;
  p.xs_c = plane; p.xs_n = c.G * p.Cg * plane;
  p.os_o = plane; p.os_n = c.G * p.Og * plane;
  if ((int64_t)(fwd ? plan->x_elems : plan->out_elems) >= (1ll << 31)) return false;
  const int T = c.KH * c.KW;
  // weights as they lie in memory when they are W[g][o][c][taps] with 8 | Cg (16-byte pieces), else a packed copy
  const bool natural = (c.KW == 1 || c.ws_kw == 1) && (c.KH == 1 || c.ws_kh == c.KW) && c.ws_c == T && (c.Cg & 7) == 0;
  p.w_mode = natural ? (fwd ? 1 : 2) : 0;
  p.ws_g = c.ws_g; p.ws_o = c.ws_o; p.ws_c = c.ws_c;
  if (p.w_mode == 2 && (c.Cg & 7)) return false;
  p.TR = TR;
  p.tpi = (c.Ho + TR - 1) / TR;
  p.n_tiles = c.N * p.tpi;
  p.n_nblocks = (p.Og + kBN - 1) / kBN;
  p.n_slots = TR + c.KH - 1;
  p.Wp = c.Wi + c.KW - 1;
  p.vpr = (c.Wi + 3) / 4;
  p.x_items = (kKC / 8) * p.n_slots * p.vpr;
  if (p.x_items > kMaxXI * kThreads) return false;
  if ((TR * c.Wo + 15) / 16 > kWaves * kMaxTM) return false;
  p.cg_stride = p.n_slots * p.Wp;
  p.lds_xbuf = (kKC / 8) * p.cg_stride * 16;
  p.n_xbuf = 1;                                  // (rows_grid takes a second buffer when a workgroup walks several tiles)
  p.lds_w_off = p.lds_xbuf;
  p.lds_bytes = p.lds_w_off + T * kBN * kWRow * 2;
  if (p.lds_bytes > kLdsLimit) return false;
  p.out_bf16 = plan->out_dtype == SYNO_BF16;
  p.m_wo = magic_of(c.Wo); p.m_vpr = magic_of(p.vpr); p.m_pcg = magic_of((int64_t)p.n_slots * p.vpr); p.m_tpi = magic_of(p.tpi);
  // the magic quotients are exact while numerator * divisor < 2^32
  if ((int64_t)kMaxXI * kThreads * p.n_slots * p.vpr >= (1ll << 32) || (int64_t)p.n_tiles * p.tpi >= (1ll << 32)) return false;
  return true;
}

// Workgroups per (group, channel block) pair: as many as there are tiles while that keeps the launch within a few
// workgroups per compute unit; beyond that a workgroup walks over several tiles and stages its weights once.
void rows_grid(RowsParams& p) {
  const int pairs = p.G * p.n_nblocks;
  const int w_bytes = p.lds_bytes - p.lds_xbuf;
  auto split = [&](int lds) { return std::min(p.n_tiles, std::max(1, 256 * std::min(kLdsLimit / lds, 4) / pairs)); };
  p.S = split(p.lds_bytes);
  if (p.S < p.n_tiles && 2 * p.lds_xbuf + w_bytes <= kLdsLimit) {
    // several tiles per workgroup: the next tile's rows are written into a second buffer while this one is read
    p.n_xbuf = 2;
    p.lds_w_off = 2 * p.lds_xbuf;
    p.lds_bytes = p.lds_w_off + w_bytes;
    p.S = split(p.lds_bytes);
  }
}

// Rough duration estimate (arbitrary units) of a tile size: bytes the launch moves through the compute units'
// load paths, the 16-pixel row tiles wasted at ragged ends, and how evenly the tiles fill the device.
double rows_cost(const RowsParams& p, int KH, int KW) {
  const int pairs = p.G * p.n_nblocks, T = KH * KW;
  const double x_bytes = (double)pairs * p.n_tiles * p.x_items * 64.0;
  const double w_bytes = (double)pairs * p.S * T * kBN * kKC * 2.0;
  const double out_bytes = (double)p.N * p.G * p.Og * p.Ho * p.Wo * (p.out_bf16 ? 2.0 : 4.0);
  double tiles16 = 0;
  for (int t = 0; t < p.tpi; ++t) tiles16 += (std::min(p.TR, p.Ho - t * p.TR) * p.Wo + 15) / 16;
  const double mfma = (double)pairs * p.N * tiles16 * 4 * T * (kKC / 32) * 16.0 / 4.0;    // SIMD cycles, summed
  const int wgs = pairs * p.S;
  const double waves_of_wgs = std::ceil((double)wgs / (256.0 * std::max(1, std::min(4, kLdsLimit / p.lds_bytes))));
  const double per_wg_tiles = std::ceil((double)p.n_tiles / p.S);
  const double mem = (x_bytes * 0.5 + w_bytes * 0.5 + out_bytes) / 256.0 / 16.0;     // cycles per CU at ~16 B/clk
  const double cmp = mfma / 256.0;
  return std::max(mem, cmp) * (wgs < 256 ? 256.0 / wgs : 1.0) + waves_of_wgs * 3000.0 + per_wg_tiles * 800.0;
}

}  // namespace

bool rows_supports(const syno_plan* plan, int which) {
  RowsParams p;
  for (int TR = 1; TR <= plan->conv.Ho; ++TR)
    if (rows_fill(plan, which, TR, p)) return true;
  return false;
}

// Picks the tile size and fills launch[which]; false when the kernel cannot take the pass.
bool rows_configure(syno_plan* plan, int which) {
  const ConvLike& c = plan->conv;
  RowsParams best{}, p;
  double best_cost = 1e300;
  for (int TR = 1; TR <= c.Ho; ++TR) {
    if (plan->opt.mfma_rows > 0 && TR != plan->opt.mfma_rows) continue;
    if (!rows_fill(plan, which, TR, p)) continue;
    rows_grid(p);
    const double cost = rows_cost(p, c.KH, c.KW);
    if (cost < best_cost) { best_cost = cost; best = p; }
  }
  if (best_cost >= 1e300) return false;
  Launch& L = plan->launch[which];
  static_assert(sizeof(RowsParams) <= sizeof(L.params), "parameter record does not fit");
  memcpy(L.params, &best, sizeof best);
  L.params_ready = true;
  L.variant = -1;       // (marks the row-streaming kernel among the family's launch records)
  const int T = c.KH * c.KW;
  L.workspace = best.w_mode == 0 ? (size_t)best.G * best.n_nblocks * T * kBN * kWRow * 2 : 0;
  return true;
}

std::string rows_describe(const syno_plan* plan, int which) {
  RowsParams p;
  memcpy(&p, plan->launch[which].params, sizeof p);
  char b[256];
  snprintf(b, sizeof b, "row-streaming rows/block=%d BN=%d tiles=%d weights=%s grid=%d tiles/workgroup=%d lds=%dB x-buffers=%d",
           p.TR, kBN, p.n_tiles * p.G * p.n_nblocks, p.w_mode ? "direct" : "packed", p.G * p.n_nblocks * p.S,
           (p.n_tiles + p.S - 1) / p.S, p.lds_bytes, p.n_xbuf);
  return b;
}

namespace {
template <int KH, int KW>
void rows_launch_window(const RowsParams& p, const uint16_t* X, const uint16_t* W, void* out, hipStream_t s) {
  auto kernel = conv_rows_bf16<KH, KW>;
  static const hipError_t lds_opt_in =
      hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsLimit);
  if (lds_opt_in != hipSuccess) return;
  hipLaunchKernelGGL(kernel, dim3(p.G * p.n_nblocks * p.S), dim3(kThreads), p.lds_bytes, s, p, X, W, out);
}
}  // namespace

syno_status launch_rows(const syno_plan* plan, int which, const void* A, const void* B, void* out, void* ws,
                        hipStream_t stream) {
  RowsParams p;
  memcpy(&p, plan->launch[which].params, sizeof p);
  const ConvLike& c = plan->conv;
  const uint16_t* weights = static_cast<const uint16_t*>(B);
  if (p.w_mode == 0) {
    if (!ws) return SYNO_ERR_WORKSPACE;
    const int T = c.KH * c.KW;
    const int64_t pieces = (int64_t)p.G * p.n_nblocks * T * kBN * (kWRow / 8);
    const bool fwd = which == SYNO_FWD;
    // the adjoint exchanges the channel roles and reverses the taps
    const int64_t w_base = fwd ? 0 : (int64_t)(c.KH - 1) * c.ws_kh + (int64_t)(c.KW - 1) * c.ws_kw;
    hipLaunchKernelGGL(rows_pack_weight, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, stream, weights,
                       static_cast<uint4*>(ws), pieces, p.G, p.n_nblocks, T, c.KW, p.Og, p.Cg, w_base, c.ws_g,
                       fwd ? c.ws_o : c.ws_c, fwd ? c.ws_c : c.ws_o, fwd ? c.ws_kh : -c.ws_kh, fwd ? c.ws_kw : -c.ws_kw);
    weights = static_cast<const uint16_t*>(ws);
  }
  const uint16_t* X = static_cast<const uint16_t*>(A);
  if (c.KH == 3 && c.KW == 3) rows_launch_window<3, 3>(p, X, weights, out, stream);
  else if (c.KH == 3) rows_launch_window<3, 1>(p, X, weights, out, stream);
  else if (c.KW == 3) rows_launch_window<1, 3>(p, X, weights, out, stream);
  else rows_launch_window<1, 1>(p, X, weights, out, stream);
  return hipGetLastError() == hipSuccess ? SYNO_OK : SYNO_ERR_HIP;
}

}  // namespace syno
