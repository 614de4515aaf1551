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
  int32_t w_mode;                       // 1: forward; 2: the adjoint (channel roles exchanged, taps reversed)
  int32_t w_packed;                     // the weights come from a copy in W[g][o][c][taps] layout in the workspace
  int32_t ws_g, ws_o, ws_c;             // element strides of that layout: group, forward output channel, input channel
  int32_t TR, tpi, n_tiles;             // output rows per tile, tiles per image, N*tpi
  int32_t n_nblocks, S;                 // 64-channel blocks per group; workgroups per (group, block) pair
  int32_t n_slots, Wp, vpr, x_items;    // row slots per tile, slot pitch (pixels), staging items per row, items per tile
  int32_t cg_stride;                    // 16-byte units between channel octets: n_slots*Wp
  int32_t lds_xbuf, n_xbuf, lds_w_off, lds_bytes;
  int32_t out_bf16;
  int32_t vec_store;                    // every result quad of 4 pixels is whole and aligned
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

// Any weight layout -> W[g][o][c][taps] contiguous with the channels padded to a multiple of 8 by zeros (the layout
// the contraction kernel reads in 16-byte pieces).  One thread per element.
__global__ __launch_bounds__(256) void rows_pack_weight(const uint16_t* __restrict__ Wt, uint16_t* __restrict__ packed,
                                                        int64_t n, int Og, int Cg, int Cgp, int KH, int KW, int ws_g,
                                                        int ws_o, int ws_c, int ws_kh, int ws_kw) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  int64_t r = i;
  const int kw = (int)(r % KW); r /= KW;
  const int kh = (int)(r % KH); r /= KH;
  const int c = (int)(r % Cgp); r /= Cgp;
  const int o = (int)(r % Og);
  const int g = (int)(r / Og);
  packed[i] = c < Cg ? Wt[(int64_t)g * ws_g + (int64_t)o * ws_o + (int64_t)c * ws_c + kh * ws_kh + kw * ws_kw] : (uint16_t)0;
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
// fp32 -> bf16 pair, round to nearest even (the hardware's conversion)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// A launch of this kernel lasts a few microseconds and a wave executes every instruction once, so the instruction
// count of the set-up and of the result stores weighs as much as the matrix work: everything that does not depend
// on the lane is kept in scalars, addresses are a uniform base plus a 32-bit lane offset, and the common case (whole
// 16-byte quads, all 64 channels present) has its own straight path.
template <int KH, int KW, bool OUTBF>
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
  const int sh = p.h_wrap ? (p.h_shift + p.h_shift_g * g) % p.Hi : 0;     // this group's cyclic row offset, < Hi
  const bool tail = (p.Cg & 7) != 0;             // the last channel octet is incomplete (packed weights only)

  // ---- what this thread stages per tile: items of 4 adjacent pixels of one input row x 8 channels
  int x_slot[kMaxXI], x_lds[kMaxXI], x_nj[kMaxXI];
  uint32_t x_src[kMaxXI];        // byte offset of (channel octet, column) inside the group's part of the tensor
#pragma unroll
  for (int k = 0; k < kMaxXI; ++k) {
    const int idx = tid + k * kThreads;
    const int cg = fdiv(idx, p.m_pcg), rem = idx - cg * (p.n_slots * p.vpr);
    const int s = fdiv(rem, p.m_vpr), x = min((rem - s * p.vpr) * 4, p.Wi - 4);   // a row's last item ends with the row
    x_slot[k] = (idx < p.x_items && cg * 8 < p.Cg) ? s : -1;      // (octets the group does not have stay zero in LDS)
    x_src[k] = (uint32_t)(cg * 8 * p.xs_c + x) * 2u;
    x_nj[k] = min(8, p.Cg - cg * 8);
    x_lds[k] = (cg * p.n_slots + s) * p.Wp + x + p.pw;            // 16-byte units
  }
  const char* Xg = reinterpret_cast<const char*>(X + (int64_t)g * p.Cg * p.xs_c);

  uint2 xr[kMaxXI][8];
  uint32_t x_ok = 0;       // bit k: item k of the tile in flight has a source row
  // requests the input rows of tile mb: every load is issued unconditionally (what has no source reads the group's
  // first elements and is replaced by zeros on its way into LDS)
  auto fetch = [&](int mb) {
    const int n = fdiv(mb, p.m_tpi), h0 = (mb - n * p.tpi) * p.TR;
    const int rows = min(p.TR, p.Ho - h0);
    const uint32_t img = (uint32_t)(n * p.xs_n) * 2u;
    x_ok = 0;
#pragma unroll
    for (int k = 0; k < kMaxXI; ++k) {
      const int s = x_slot[k];
      int r;
      bool ok;
      if (p.h_wrap) {
        r = h0 + s + sh;
        r = r >= p.Hi ? r - p.Hi : r;
        ok = (unsigned)s < (unsigned)rows;
      } else {
        r = h0 - p.ph + s;
        ok = s >= 0 && s < rows + KH - 1 && (unsigned)r < (unsigned)p.Hi;
      }
      x_ok |= ok ? (1u << k) : 0u;
      const uint32_t o = ok ? img + x_src[k] + (uint32_t)(r * p.Wi) * 2u : 0u;
      const uint32_t step = ok ? (uint32_t)p.xs_c * 2u : 0u;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint32_t oj = o + step * (uint32_t)(tail ? min(j, x_nj[k] - 1) : j);
        xr[k][j] = __builtin_bit_cast(uint2, *reinterpret_cast<const bf16x4_unaligned*>(Xg + oj));
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
      if (tail) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (j >= x_nj[k]) xr[k][j] = make_uint2(0, 0);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;     // high or low halves of (second, first)
        auto w = [&](int j) { return (i >> 1) ? xr[k][j].y : xr[k][j].x; };
        uint4 v;
        v.x = __builtin_amdgcn_perm(w(1), w(0), sel);
        v.y = __builtin_amdgcn_perm(w(3), w(2), sel);
        v.z = __builtin_amdgcn_perm(w(5), w(4), sel);
        v.w = __builtin_amdgcn_perm(w(7), w(6), sel);
        xl[x_lds[k] + i] = ok ? v : make_uint4(0, 0, 0, 0);
      }
    }
  };

  int mb = s_id;
  fetch(mb);           // (S <= n_tiles: every workgroup has a first tile)

  // ---- the weight block: W[g][o][c][T taps] (as it lies in memory, or a copy a small kernel has put into that
  // layout).  A thread takes 8 channels x T taps of one forward output channel (T adjacent 16-byte loads), twice; all
  // requests go out before anything is waited for, behind the first tile's input rows.
  constexpr int kWItems = kBN * (kKC / 8) / kThreads;      // 2
  uint32_t win[kWItems][4 * T];
  int w_dst[kWItems];
  bool w_live[kWItems];
  const bool adj = p.w_mode == 2;
  {
    // forward: rows are this block's output channels; adjoint: the reduction runs over the forward output channels and
    // this block's rows are forward input channels (p.Og counts those, p.Cg the forward output channels)
    const uint16_t* Wn = Wv + (int64_t)g * p.ws_g + (int64_t)nb * kBN * (adj ? p.ws_c : p.ws_o);
#pragma unroll
    for (int it = 0; it < kWItems; ++it) {
      const int i = tid + it * kThreads;
      const int octet = i & (kKC / 8 - 1), row = i >> 3;          // (forward: 8 octets of c per row o; adjoint: 8 octets
      static_assert(kKC / 8 == 8 && kBN / 8 == 8, "index split");  //  of the block's 64 rows per forward output channel)
      w_live[it] = adj ? (row < p.Cg && nb * kBN + octet * 8 < p.Og) : (nb * kBN + row < p.Og && octet * 8 < p.Cg);
      // forward: piece index of tap 0 in [tap][o][c]; adjoint: element index of (tap T-1, row octet*8, column row)
      w_dst[it] = adj ? (octet * 8) * kWRow + row : row * (kWRow / 8) + octet;
      const uint16_t* src = Wn + (w_live[it] ? row * p.ws_o + octet * 8 * T : 0);
#pragma unroll
      for (int q = 0; q < T; ++q) {
        const u32x4_unaligned v = *reinterpret_cast<const u32x4_unaligned*>(src + q * 8);
        win[it][4 * q + 0] = v[0]; win[it][4 * q + 1] = v[1]; win[it][4 * q + 2] = v[2]; win[it][4 * q + 3] = v[3];
      }
    }
  }
  // while the requests travel: zero the input buffers once (slot edges are the window's zero padding and are never
  // written afterwards)
  {
    uint4* z = reinterpret_cast<uint4*>(smem);
    const int n16 = (p.n_xbuf * p.lds_xbuf) >> 4;
    for (int i = tid; i < n16; i += kThreads) z[i] = make_uint4(0, 0, 0, 0);
  }
  // ---- per-lane operand bases (the same for every tile): row tile t of this wave is tile wv + t*kWaves of the block
  int a_base[kMaxTM];
#pragma unroll
  for (int t = 0; t < kMaxTM; ++t) {
    int m = (wv + t * kWaves) * 16 + (lane & 15);
    if (m >= p.TR * p.Wo) m = 0;
    const int i = fdiv(m, p.m_wo), w = m - i * p.Wo;
    a_base[t] = (i * p.Wp + w + (lane >> 4) * p.cg_stride) * 16;
  }
  const int b_lane = p.lds_w_off + ((lane & 15) * kWRow + (lane >> 4) * 8) * 2;
  // LDS byte offset of the A operand at k-step ks = (tap, 32-channel half)
  int a_step[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const int tap = ks / (kKC / 32), half = ks % (kKC / 32);
    a_step[ks] = ((tap / KW) * p.Wp + (tap % KW) + half * 4 * p.cg_stride) * 16;
  }
  // result addressing: a lane holds 4 consecutive pixels (quad 4*(lane>>4) of its row tile) of channel lane&15 of a
  // 16-channel column tile
  const int m_lane = wv * 16 + 4 * (lane >> 4);
  const int o_left = p.Og - nb * kBN - (lane & 15);        // column tile u holds a channel of this lane iff 16u < o_left
  constexpr int ESZ = OUTBF ? 2 : 4;
  const uint32_t out_lane = (uint32_t)((g * p.Og + nb * kBN + (lane & 15)) * p.os_o + m_lane) * ESZ;

  if (!adj) {
    // one 16-byte piece per tap: [tap][o][c]
    uint4* wl = reinterpret_cast<uint4*>(smem + p.lds_w_off);
#pragma unroll
    for (int it = 0; it < kWItems; ++it) {
#pragma unroll
      for (int tap = 0; tap < T; ++tap) {
        uint32_t d[4];
#pragma unroll
        for (int h = 0; h < 4; ++h) {
          // channels 2h and 2h+1 of this tap: elements (2h)*T+tap and (2h+1)*T+tap of the 8*T loaded ones
          const int e0 = (2 * h) * T + tap, e1 = (2 * h + 1) * T + tap;
          const uint32_t sel = ((e0 & 1) ? 0x0302u : 0x0100u) | ((e1 & 1) ? 0x07060000u : 0x05040000u);
          d[h] = __builtin_amdgcn_perm(win[it][e1 >> 1], win[it][e0 >> 1], sel);
        }
        wl[tap * (kBN * kWRow / 8) + w_dst[it]] = w_live[it] ? make_uint4(d[0], d[1], d[2], d[3]) : make_uint4(0, 0, 0, 0);
      }
    }
  } else {
    // the adjoint's B operand out of the same memory, taps reversed: element (o, c, tap) goes to [T-1-tap][c][o]
    uint16_t* wl = reinterpret_cast<uint16_t*>(smem + p.lds_w_off);
#pragma unroll
    for (int it = 0; it < kWItems; ++it) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int tap = 0; tap < T; ++tap) {
          const int e = j * T + tap;
          const uint32_t v = w_live[it] ? win[it][e >> 1] : 0u;
          wl[((T - 1 - tap) * kBN + j) * kWRow + w_dst[it]] = (uint16_t)((e & 1) ? v >> 16 : v);
        }
    }
  }
  __syncthreads();     // the zero fill is complete before any input row is staged over it

  int buf = 0;
  for (; mb < p.n_tiles; mb += p.S) {
    const int n = fdiv(mb, p.m_tpi), h0 = (mb - n * p.tpi) * p.TR;
    const int rows = min(p.TR, p.Ho - h0);
    const int block_px = rows * p.Wo;
    stage(buf);
    __syncthreads();     // this tile's rows (and, first time, the weights) are in LDS; every wave has left the tile
                         // before, whose buffer the tile after this one will overwrite
    if (mb + p.S < p.n_tiles) fetch(mb + p.S);
    const int MT = (block_px + 15) >> 4;
    const int my_tiles = wv < MT ? (MT - wv + kWaves - 1) / kWaves : 0;
    const int xoff = buf * p.lds_xbuf;
    char* const out_tile = reinterpret_cast<char*>(out) + ((int64_t)n * p.os_n + (int64_t)h0 * p.Wo) * ESZ;

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
        for (int u = 0; u < 4; ++u)
          b[u] = *reinterpret_cast<const uint4*>(smem + b_lane + u * (16 * kWRow * 2) + tap * B_TAP + half * 64);
        const int a_off = xoff + a_step[ks];
#pragma unroll
        for (int t = 0; t < NTL; ++t) a[t] = *reinterpret_cast<const uint4*>(smem + a_base[t] + a_off);
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
        // issue order: one LDS read of the next k-step after each of the first MFMAs of this one, so that the
        // fragments are in flight under the matrix work instead of being waited for right after their request
        if constexpr (ks + 1 < KS) {
          constexpr int NR = NTL + 4, NM = NTL * 4, NP = NR < NM ? NR : NM;
#pragma unroll
          for (int i = 0; i < NP; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // LDS read
          }
          if constexpr (NR > NP) __builtin_amdgcn_sched_group_barrier(0x100, NR - NP, 0);
          if constexpr (NM > NP) __builtin_amdgcn_sched_group_barrier(0x008, NM - NP, 0);
        }
        __builtin_amdgcn_sched_barrier(0);   // nothing moves across k-steps
      };
      read(std::integral_constant<int, 0>{}, fa[0], fb[0]);
      auto steps = [&](auto self, auto ks_c) -> void {      // k-steps 0 .. KS-1, unrolled at compile time
        constexpr int ks = decltype(ks_c)::value;
        step(ks_c);
        if constexpr (ks + 1 < KS) self(self, std::integral_constant<int, ks + 1>{});
      };
      steps(steps, std::integral_constant<int, 0>{});

      // ---- store.  Element (t, u, j) of this lane is pixel m_lane + 64t + j of channel 16u + lane&15.
#pragma unroll
      for (int t = 0; t < NTL; ++t) {
        const int m0 = m_lane + t * 64;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (u * 16 >= o_left || m0 >= block_px) continue;
          char* dst = out_tile + (int64_t)(t * 64 + u * 16 * p.os_o) * ESZ + out_lane;
          if (p.vec_store) {       // every quad is whole and 16-byte (8-byte for bf16) aligned
            if constexpr (OUTBF)
              *reinterpret_cast<uint2*>(dst) = make_uint2(pack_bf16x2(acc[t][u][0], acc[t][u][1]), pack_bf16x2(acc[t][u][2], acc[t][u][3]));
            else
              *reinterpret_cast<floatx4*>(dst) = acc[t][u];
          } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (m0 + j < block_px) {
                if constexpr (OUTBF) reinterpret_cast<uint16_t*>(dst)[j] = (uint16_t)pack_bf16x2(acc[t][u][j], 0.f);
                else reinterpret_cast<float*>(dst)[j] = acc[t][u][j];
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
  const bool natural = (c.KW == 1 || c.ws_kw == 1) && (c.KH == 1 || c.ws_kh == c.KW) && c.ws_c == T && (c.Cg & 7) == 0 &&
                       (c.G == 1 || c.ws_g >= 0) && c.ws_o >= 0;
  p.w_mode = fwd ? 1 : 2;
  p.w_packed = natural ? 0 : 1;
  const int Cgp = (c.Cg + 7) & ~7;
  p.ws_c = T;
  p.ws_o = natural ? c.ws_o : Cgp * T;
  p.ws_g = natural ? c.ws_g : c.Og * Cgp * T;
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
  p.vec_store = (c.Ho * c.Wo) % 4 == 0 && (TR * c.Wo) % 4 == 0;
  if ((int64_t)(fwd ? plan->out_elems : plan->x_elems) * (p.out_bf16 ? 2 : 4) >= (1ll << 32)) return false;   // 32-bit lane offsets
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

// Order of preference among tile sizes, from measurements on the benchmark shapes: whole aligned result quads
// (16-byte stores) before anything else; then one tile per workgroup (every load of the launch is requested at
// once); then few, large tiles (the weight block is staged once per workgroup).  Smaller is better.
double rows_cost(const RowsParams& p) {
  const double tiles_per_wg = std::ceil((double)p.n_tiles / p.S);
  const int wgs = p.G * p.n_nblocks * p.S;
  return (p.vec_store ? 0.0 : 1e6) + (tiles_per_wg - 1.0) * 1e4 + (wgs < 96 ? (96 - wgs) * 10.0 : 0.0) + wgs * 1e-3;
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
    const double cost = rows_cost(p);
    if (cost < best_cost) { best_cost = cost; best = p; }
  }
  if (best_cost >= 1e300) return false;
  // a workgroup that walks over several tiles is not yet faster than the tiled kernel of this family: leave those
  // shapes there unless this kernel is named explicitly
  if (best.S < best.n_tiles && plan->opt.mfma_variant != -1) return false;
  Launch& L = plan->launch[which];
  static_assert(sizeof(RowsParams) <= sizeof(L.params), "parameter record does not fit");
  memcpy(L.params, &best, sizeof best);
  L.params_ready = true;
  L.variant = -1;       // (marks the row-streaming kernel among the family's launch records)
  const int T = c.KH * c.KW;
  L.workspace = best.w_packed ? (size_t)c.G * c.Og * ((c.Cg + 7) & ~7) * T * 2 : 0;
  return true;
}

std::string rows_describe(const syno_plan* plan, int which) {
  RowsParams p;
  memcpy(&p, plan->launch[which].params, sizeof p);
  char b[256];
  snprintf(b, sizeof b, "row-streaming rows/block=%d BN=%d tiles=%d weights=%s grid=%d tiles/workgroup=%d lds=%dB x-buffers=%d",
           p.TR, kBN, p.n_tiles * p.G * p.n_nblocks, p.w_packed ? "packed" : "direct", p.G * p.n_nblocks * p.S,
           (p.n_tiles + p.S - 1) / p.S, p.lds_bytes, p.n_xbuf);
  return b;
}

namespace {
template <int KH, int KW, bool OUTBF>
void rows_launch_typed(const RowsParams& p, const uint16_t* X, const uint16_t* W, void* out, hipStream_t s) {
  auto kernel = conv_rows_bf16<KH, KW, OUTBF>;
  static const hipError_t lds_opt_in =
      hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsLimit);
  if (lds_opt_in != hipSuccess) return;
  hipLaunchKernelGGL(kernel, dim3(p.G * p.n_nblocks * p.S), dim3(kThreads), p.lds_bytes, s, p, X, W, out);
}
template <int KH, int KW>
void rows_launch_window(const RowsParams& p, const uint16_t* X, const uint16_t* W, void* out, hipStream_t s) {
  if (p.out_bf16) rows_launch_typed<KH, KW, true>(p, X, W, out, s);
  else rows_launch_typed<KH, KW, false>(p, X, W, out, s);
}
}  // namespace

syno_status launch_rows(const syno_plan* plan, int which, const void* A, const void* B, void* out, void* ws,
                        hipStream_t stream) {
  RowsParams p;
  memcpy(&p, plan->launch[which].params, sizeof p);
  const ConvLike& c = plan->conv;
  const uint16_t* weights = static_cast<const uint16_t*>(B);
  if (p.w_packed) {
    if (!ws) return SYNO_ERR_WORKSPACE;
    const int Cgp = (c.Cg + 7) & ~7;
    const int64_t n = (int64_t)c.G * c.Og * Cgp * c.KH * c.KW;
    hipLaunchKernelGGL(rows_pack_weight, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, weights,
                       static_cast<uint16_t*>(ws), n, c.Og, c.Cg, Cgp, c.KH, c.KW, c.ws_g, c.ws_o, c.ws_c, c.ws_kh, c.ws_kw);
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
