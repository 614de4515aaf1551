// MFMA backward-weight contraction for convolution-like operators (bf16 or fp32 inputs, fp32 result):
//   dW[g,o,c,kh,kw] = sum_{n,h,w} G[n, g*Og+o, h, w] * X[n, g*Cg+c, row(h,g)+kh-ph, w+kw-pw]
// Kernels in this file:
//   dw_mfma_bf16, dw_mfma_f32   any supported window; the source rows of a chunk come from a table in LDS
//   dw_rows_f32, dw_rows_bf16   windows with a row extent (KH = 3): eight waves in two halves that alternate between
//                               multiplying one LDS buffer and staging the next chunk into the other
//   dw_reduce_slots, _tiles     fixed-order sum of the split partials into dW
// A GEMM per group and tap with M = o, N = c and the reduction over the pixels (n,h,w), which is the
// contiguous axis of both operands - exactly what the bf16 MFMA wants (8 consecutive K per lane).
//
// Both operands are staged pixel-contiguous into LDS, rows laid out with a pitch of W plus at least
// one zero column: that column is the zero padding of the window on either side, so a tap is a pure
// shift of the X index by (kw - pw) elements and needs no mask.  G has zeros in its pad columns, so
// whatever X holds there never contributes.  A shifted 8-element fragment is cut out of two aligned
// 16-byte LDS reads with v_alignbit.  With a window along h as well (KH = 3) a chunk of rows stays inside
// one image, X is staged with its KH-1 halo rows (zero outside the image), the row pitch is a multiple of
// 8 elements, and tap kh is a further shift by kh whole rows.
//
// The pixel axis is split over workgroups (split-K); each writes its tile of sums into the workspace in
// the register layout of the accumulators (coalesced 16-byte stores) and a second kernel adds the partials
// in a fixed order and scatters them into dW, so the result does not depend on scheduling.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <cstdio>
#include <cstring>
#include <string>
#include <type_traits>

#include "plan.h"

namespace syno {

struct DwParams {
  int32_t G, Og, Cg, H, W, KH, KW, ph, pw;
  int32_t rows_total;                  // N*H
  int32_t h_wrap, h_shift, h_shift_g;  // X row = (h + h_shift + h_shift_g*g) mod H when wrapped, else h
  int32_t plane, gs_n, xs_n;           // H*W; image strides of G and X
  int32_t ws_g, ws_o, ws_c, ws_kh, ws_kw;   // dW strides
  int32_t w_elems;                     // elements of dW
  int32_t n_tiles, ct, slots;          // workgroup tiles (g, o block, c block); c-tiles per wave; 8 * ct * KH*KW
  int32_t pitch, TRK, CP, CPp;         // LDS row pitch, rows per chunk, chunk length (multiple of 32), LDS channel pitch
  int32_t CPg;                         // fp32 kernel: channel pitch of the G tile (it has no halo rows); CPp is X's
  int32_t rows_per_split, n_splits, n_oblk, n_cblk;
  int32_t n_xrows;                     // rows of X staged per chunk: TRK + KH - 1
  int32_t cpi;                         // KH > 1: chunks per image (chunks do not cross images); else 0
  int32_t ipc, n_images;               // bf16, KH > 1, cpi == 1: whole images per chunk, each with its own halo rows
  int32_t chunks_per_split, n_chunks;
  int32_t items;                       // 64 * n_xrows * W/2 dword items per tensor per chunk
  uint32_t magic_w2, magic_rw2;        // ceil(2^32/d) for d = items per row and n_xrows * items per row (0 for d = 1)
  int32_t lds_x_off, lds_tab_off, lds_bytes;
  // fp32 kernel for windows with a row extent (chunks inside one image, source rows affine in the staged row):
  int32_t direct;                      // that kernel takes this plan
  int32_t ni_g, ni_x;                  // staging items per thread of G and of X
  int32_t mode;                        // pixels per staging item: 4, 2, 1, or a whole row of 7 or 14
  int32_t lds_buf;                     // bytes of one LDS buffer (G tile, then X tile at lds_x_off); there are two
  uint32_t magic_cpi;                  // ceil(2^32/d) for d = cpi (0 for d = 1); magic_w2 is for the items per row
};

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
constexpr int kGuard = 8;     // zero elements in front of each X channel row (a tap may reach one element back)
// staging items per thread, tensor and chunk (256 threads): 26-28 of one or two pixels (a dword), or 18 of four (two
// dwords) - about the same registers either way
constexpr int dw_items(int ep) { return ep == 4 ? 18 : ep == 2 ? 28 : 32; }   // (28: a whole 14 x 14 image with its halo rows; 32: two 7 x 7 images)

__device__ __forceinline__ uint32_t alignbit16(uint32_t hi, uint32_t lo) { return __builtin_amdgcn_alignbit(hi, lo, 16); }

// Elements [s, s+8) of the 16 elements held in two consecutive aligned groups (lo, hi), s in 0..8.
template <int S>
__device__ __forceinline__ bf16x8 cut(const uint4& lo, const uint4& hi) {
  const uint32_t d[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
  uint4 r;
  if constexpr (S % 2 == 0) {
    r = make_uint4(d[S / 2], d[S / 2 + 1], d[S / 2 + 2], d[S / 2 + 3]);
  } else {
    r = make_uint4(alignbit16(d[S / 2 + 1], d[S / 2]), alignbit16(d[S / 2 + 2], d[S / 2 + 1]),
                   alignbit16(d[S / 2 + 3], d[S / 2 + 2]), alignbit16(d[S / 2 + 4], d[S / 2 + 3]));
  }
  return __builtin_bit_cast(bf16x8, r);
}

template <int KH, int KW, int CT>
__device__ __forceinline__ void dw_finish(const DwParams& p, float* __restrict__ partial, int g, int ob, int cb, int split,
                                          int widx, int lane, const floatx4 (&acc)[2][CT][KH * KW]);

// The k-steps of one staged chunk of the bf16 kernels: 32 pixels each; the LDS reads of the next step are issued before
// the MFMAs of the current one.  `gp` and `xp` are the channel pitches (elements) of the G and the X tile.
template <int KH, int KW, int CT>
__device__ __forceinline__ void dw_bf16_chunk(const DwParams& p, const uint16_t* gl, const uint16_t* xl,
                                              const int (&a_base)[2], const int (&b_base)[CT],
                                              floatx4 (&acc)[2][CT][KH * KW]) {
  const int steps = p.CP >> 5;
  constexpr int NX = KW == 1 ? 2 : 3;      // 16-byte groups of X read per (c-tile, kh)
  struct Frags { uint4 a[2]; uint4 x[CT * KH][NX]; };
  auto read = [&](int st, Frags& f) {
#pragma unroll
    for (int i = 0; i < 2; ++i) f.a[i] = *reinterpret_cast<const uint4*>(gl + a_base[i] + st * 32);
#pragma unroll
    for (int i = 0; i < CT; ++i)
#pragma unroll
      for (int kh = 0; kh < KH; ++kh) {
        const uint16_t* xp = xl + b_base[i] + st * 32 + kh * p.pitch;
#pragma unroll
        for (int q = 0; q < NX; ++q) f.x[i * KH + kh][q] = *reinterpret_cast<const uint4*>(xp + 8 * q);
      }
  };
  // tap (kh, kw) reads X shifted by kh rows and (kw - pw) elements: element 8 + kw - pw of the groups read at
  // row offset kh*pitch (a multiple of 8 elements when KH > 1)
  auto mfmas = [&](const Frags& f) {
#pragma unroll
    for (int i = 0; i < CT; ++i)
#pragma unroll
      for (int kh = 0; kh < KH; ++kh) {
        const uint4(&x)[NX] = f.x[i * KH + kh];
        bf16x8 b[KW];
        if constexpr (KW == 1) {
          b[0] = cut<8>(x[0], x[1]);
        } else {
          b[0] = cut<7>(x[0], x[1]);
          b[1] = cut<8>(x[0], x[1]);
          b[2] = cut<1>(x[1], x[2]);     // one more element to the right reaches into the third group
        }
#pragma unroll
        for (int t = 0; t < KW; ++t)
#pragma unroll
          for (int ao = 0; ao < 2; ++ao)
            acc[ao][i][kh * KW + t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, f.a[ao]), b[t],
                                                                             acc[ao][i][kh * KW + t], 0, 0, 0);
      }
  };
  Frags f0, f1;
  read(0, f0);
  int st = 0;
  for (; st + 2 < steps; st += 2) {
    read(st + 1, f1); mfmas(f0);
    read(st + 2, f0); mfmas(f1);
  }
  if (st + 1 < steps) { read(st + 1, f1); mfmas(f0); mfmas(f1); }
  else mfmas(f0);
}

// One workgroup: group g, 64 output channels x 32*CT input channels, one split of the pixel rows.
// 4 waves; wave (wo, wc) owns o-tiles {2wo, 2wo+1} x CT c-tiles x KH*KW taps (CT = 2 for up to 3 taps, 1 for 9).
// Staging moves items of EP adjacent pixels of a row: 4 (two dwords) when W is a multiple of 4, else 2, else 1.
template <int KH, int KW, int CT, int EP>
__global__ __launch_bounds__(256) void dw_mfma_bf16(const DwParams p, const uint16_t* __restrict__ Gt,
                                                    const uint16_t* __restrict__ Xt, float* __restrict__ partial) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* gl = reinterpret_cast<uint16_t*>(smem);                 // [64][CPp]
  uint16_t* xl = reinterpret_cast<uint16_t*>(smem + p.lds_x_off);   // [32*CT][CPp], data starts at kGuard
  int* row_tab = reinterpret_cast<int*>(smem + p.lds_tab_off);      // [2][n_xrows]: G row offset, X row offset (-1: none)

  const int tid = threadIdx.x, lane = tid & 63;
  const int widx = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wo = widx >> 1, wc = widx & 1;
  int bid = blockIdx.x;
  const int split = bid % p.n_splits; bid /= p.n_splits;
  const int cb = bid % p.n_cblk; bid /= p.n_cblk;
  const int ob = bid % p.n_oblk;
  const int g = bid / p.n_oblk;
  const int chunk_begin = split * p.chunks_per_split;
  const int chunk_end = min(p.n_chunks, chunk_begin + p.chunks_per_split);
  constexpr int CX = 32 * CT;      // X channels of this workgroup
  constexpr int T = KH * KW;

  // zero both tiles once: pad columns, guards and tails stay zero for the whole kernel
  {
    uint4* z = reinterpret_cast<uint4*>(smem);
    const int n16 = p.lds_tab_off >> 4;
    for (int i = tid; i < n16; i += 256) z[i] = make_uint4(0, 0, 0, 0);
  }
  // per-thread item descriptors, the same for G and X: (channel, row, dword) of the chunk
  // goff: element offset inside the 64-channel slab, shifted left by one; bit 0 set = G channel beyond Og
  // meta: LDS element offset | row << 20 | (X channel beyond Cg) << 30 ; -1 when unused
  constexpr int kDwItems = dw_items(EP);
  constexpr int EPW = EP == 4 ? 2 : 1;    // dwords per item
  int it_goff[kDwItems], it_meta[kDwItems];
  const int W2 = p.W / EP;                // items per row
  const int o_lim = p.Og - ob * 64, c_lim = min(p.Cg - cb * CX, CX);     // channels beyond are zero
#pragma unroll
  for (int k = 0; k < kDwItems; ++k) {
    const int idx = tid + k * 256;
    const int ch = __umulhi((uint32_t)idx, p.magic_rw2);
    const int rem = idx - ch * (p.n_xrows * W2);
    const int r = p.magic_w2 ? __umulhi((uint32_t)rem, p.magic_w2) : rem;   // (one item per row: no division)
    const int j = rem - r * W2;
    it_goff[k] = ((ch * p.plane + EP * j) << 1) | (ch < o_lim ? 0 : 1);
    it_meta[k] = idx < p.items ? ((ch * p.CPp + r * p.pitch + EP * j) | (r << 20) | (ch < c_lim ? 0 : (1 << 30))) : -1;
  }
  const uint16_t* Gg = Gt + (int64_t)(g * p.Og + ob * 64) * p.plane;
  const uint16_t* Xg = Xt + (int64_t)(g * p.Cg + cb * CX) * p.plane;

  floatx4 acc[2][CT][T];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < CT; ++b)
#pragma unroll
      for (int t = 0; t < T; ++t) acc[a][b][t] = floatx4{0.f, 0.f, 0.f, 0.f};

  // operand bases (element indices)
  int a_base[2], b_base[CT];
#pragma unroll
  for (int a = 0; a < 2; ++a) a_base[a] = ((2 * wo + a) * 16 + (lane & 15)) * p.CPp + (lane >> 4) * 8;
#pragma unroll
  for (int b = 0; b < CT; ++b) b_base[b] = ((CT * wc + b) * 16 + (lane & 15)) * p.CPp + (lane >> 4) * 8 + kGuard - 8;

  uint32_t gr[kDwItems][EPW], xr[kDwItems][EPW];
  for (int q = chunk_begin; q < chunk_end; ++q) {
    __syncthreads();        // previous chunk fully consumed (and, first time, the zero fill is complete)
    if (tid < p.n_xrows) {
      int go = -1, xo = -1;
      if (KH == 1) {
        // rows of any image, cyclic row shift allowed: G row rho <-> X row (h + shift) mod H of the same image
        const int rho = q * p.TRK + tid;
        if (rho < p.rows_total) {
          const int n = rho / p.H, h = rho - n * p.H;
          const int r = p.h_wrap ? (h + p.h_shift + p.h_shift_g * g) % p.H : h;
          go = n * p.gs_n + h * p.W;
          xo = n * p.xs_n + r * p.W;
        }
      } else {
        if (p.ipc > 1) {
          // several whole images, each in H + KH - 1 slots: slot l of an image holds G row l (the last KH - 1 stay
          // zero) and X row l - ph (zero outside the image), so a tap is the same shift of whole rows everywhere
          const int per = p.H + KH - 1;
          const int i = tid / per, l = tid - i * per;
          const int n = q * p.ipc + i;
          if (n < p.n_images) {
            if (l < p.H) go = n * p.gs_n + l * p.W;
            const int hx = l - p.ph;
            if (hx >= 0 && hx < p.H) xo = n * p.xs_n + hx * p.W;
          }
        } else {
        // rows h0 .. h0+TRK-1 of image n; X slot r holds image row h0 - ph + r (zero outside the image)
        const int n = q / p.cpi, h0 = (q - n * p.cpi) * p.TRK;
        const int rows = min(p.TRK, p.H - h0);
        if (tid < rows) go = n * p.gs_n + (h0 + tid) * p.W;
        const int hx = h0 - p.ph + tid;
        if (tid < rows + KH - 1 && hx >= 0 && hx < p.H) xo = n * p.xs_n + hx * p.W;
        }
      }
      row_tab[tid] = go;
      row_tab[p.n_xrows + tid] = xo;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kDwItems; ++k) {
#pragma unroll
      for (int w = 0; w < EPW; ++w) { gr[k][w] = 0; xr[k][w] = 0; }
      if (it_meta[k] >= 0) {
        const int r = (it_meta[k] >> 20) & 1023;
        const int go = row_tab[r], xo = row_tab[p.n_xrows + r];
        if constexpr (EP == 1) {
          if (go >= 0 && !(it_goff[k] & 1)) gr[k][0] = Gg[go + (it_goff[k] >> 1)];
          if (xo >= 0 && !(it_meta[k] >> 30)) xr[k][0] = Xg[xo + (it_goff[k] >> 1)];
        } else if constexpr (EP == 2) {
          if (go >= 0 && !(it_goff[k] & 1)) gr[k][0] = *reinterpret_cast<const uint32_t*>(Gg + go + (it_goff[k] >> 1));
          if (xo >= 0 && !(it_meta[k] >> 30)) xr[k][0] = *reinterpret_cast<const uint32_t*>(Xg + xo + (it_goff[k] >> 1));
        } else {
          if (go >= 0 && !(it_goff[k] & 1)) {
            const uint2 t = *reinterpret_cast<const uint2*>(Gg + go + (it_goff[k] >> 1));
            gr[k][0] = t.x; gr[k][EPW - 1] = t.y;
          }
          if (xo >= 0 && !(it_meta[k] >> 30)) {
            const uint2 t = *reinterpret_cast<const uint2*>(Xg + xo + (it_goff[k] >> 1));
            xr[k][0] = t.x; xr[k][EPW - 1] = t.y;
          }
        }
      }
    }
#pragma unroll
    for (int k = 0; k < kDwItems; ++k)
      if (it_meta[k] >= 0) {
        const int lo = it_meta[k] & 0xfffff;
        if constexpr (EP == 1) {
          gl[lo] = (uint16_t)gr[k][0];
          if (!(it_meta[k] >> 30)) xl[lo + kGuard] = (uint16_t)xr[k][0];   // (channels X does not have stay zero)
        } else if constexpr (EP == 2) {
          *reinterpret_cast<uint32_t*>(gl + lo) = gr[k][0];
          if (!(it_meta[k] >> 30)) *reinterpret_cast<uint32_t*>(xl + lo + kGuard) = xr[k][0];
        } else {
          *reinterpret_cast<uint2*>(gl + lo) = make_uint2(gr[k][0], gr[k][EPW - 1]);
          if (!(it_meta[k] >> 30)) *reinterpret_cast<uint2*>(xl + lo + kGuard) = make_uint2(xr[k][0], xr[k][EPW - 1]);
        }
      }
    __syncthreads();
    dw_bf16_chunk<KH, KW, CT>(p, gl, xl, a_base, b_base, acc);
  }
  dw_finish<KH, KW, CT>(p, partial, g, ob, cb, split, widx, lane, acc);
}

// The k-steps of one staged chunk: 4 pixels each; the fragments of the next step are read while the MFMAs of the
// current one issue (one wave per SIMD here, so nothing else would cover the LDS latency).
template <int KH, int KW, int CT>
__device__ __forceinline__ void dw_f32_chunk(const DwParams& p, const float* gl, const float* xl, const int (&a_base)[2],
                                             const int (&b_base)[CT], floatx4 (&acc)[2][CT][KH * KW], int first = 0,
                                             int stride = 1) {
  constexpr int T = KH * KW;
  const int steps = p.CP >> 2;
  auto read = [&](int st, float (&a)[2], float (&b)[CT * T]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) a[i] = gl[a_base[i] + st * 4];
#pragma unroll
    for (int i = 0; i < CT; ++i)
#pragma unroll
      for (int kh = 0; kh < KH; ++kh)
#pragma unroll
        for (int t = 0; t < KW; ++t) b[i * T + kh * KW + t] = xl[b_base[i] + st * 4 + kh * p.pitch + t];
  };
  auto mfmas = [&](const float (&a)[2], const float (&b)[CT * T]) {
#pragma unroll
    for (int i = 0; i < CT; ++i)
#pragma unroll
      for (int t = 0; t < T; ++t)
#pragma unroll
        for (int ao = 0; ao < 2; ++ao)
          acc[ao][i][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[ao], b[i * T + t], acc[ao][i][t], 0, 0, 0);
  };
  auto interleave = [&]() {       // (left to the compiler when a step has only a handful of MFMAs)
    if constexpr (CT * T >= 6)
#pragma unroll
    for (int i = 0; i < CT * T; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);     // 2 MFMAs
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // 1 LDS read
    }
  };
  // the wave takes steps first, first + stride, ... (waves that share an output tile split the steps between them)
  float fa0[2], fb0[CT * T], fa1[2], fb1[CT * T];
  int st = first;
  if (st >= steps) return;
  read(st, fa0, fb0);
  for (; st + 2 * stride < steps; st += 2 * stride) {
    // one fragment read of the next step after every second MFMA of the current one: the reads issue in the
    // shadow of the matrix pipe and a whole step lies between a fragment's read and its use
    read(st + stride, fa1, fb1); mfmas(fa0, fb0); interleave();
    read(st + 2 * stride, fa0, fb0); mfmas(fa1, fb1); interleave();
  }
  if (st + stride < steps) { read(st + stride, fa1, fb1); mfmas(fa0, fb0); mfmas(fa1, fb1); }
  else mfmas(fa0, fb0);
}

// Leaves the workgroup's sums: in dW itself when there is one split, else in the workspace in accumulator layout.
template <int KH, int KW, int CT>
__device__ __forceinline__ void dw_finish(const DwParams& p, float* __restrict__ partial, int g, int ob, int cb, int split,
                                              int widx, int lane, const floatx4 (&acc)[2][CT][KH * KW]) {
  constexpr int CX = 32 * CT, T = KH * KW;
  const int wo = widx >> 1, wc = widx & 1;
  // One split only (large dW, few pixels): nothing to add up, the sums go straight into dW (`partial` is dW then):
  // lane holds 4 consecutive o (rows of D) at one c (column).
  if (p.n_splits == 1) {
    float* dw = partial + (int64_t)g * p.ws_g;
#pragma unroll
    for (int ao = 0; ao < 2; ++ao)
#pragma unroll
      for (int i = 0; i < CT; ++i) {
        const int c = cb * CX + (CT * wc + i) * 16 + (lane & 15);
        if (c >= p.Cg) continue;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int o = ob * 64 + (2 * wo + ao) * 16 + 4 * (lane >> 4) + v;
          if (o >= p.Og) continue;
#pragma unroll
          for (int t = 0; t < T; ++t)
            dw[(int64_t)o * p.ws_o + (int64_t)c * p.ws_c + (t / KW) * p.ws_kh + (t % KW) * p.ws_kw] = acc[ao][i][t][v];
        }
      }
    return;
  }
  // partial[split][tile][slot][lane]: every accumulator register quadruple goes out as it is, one 16-byte store
  // per lane (1 KB per wave and slot); the reduction kernel knows which weights a (slot, lane) holds
  constexpr int SLOTS = 8 * CT * T;
  const int tile = (g * p.n_oblk + ob) * p.n_cblk + cb;
  floatx4* dst = reinterpret_cast<floatx4*>(partial) +
                 ((int64_t)split * p.n_tiles + tile) * (SLOTS * 64) + (widx * 2 * CT * T) * 64 + lane;
#pragma unroll
  for (int ao = 0; ao < 2; ++ao)
#pragma unroll
    for (int i = 0; i < CT; ++i)
#pragma unroll
      for (int t = 0; t < T; ++t) dst[((ao * CT + i) * T + t) * 64] = acc[ao][i][t];
}

// fp32 inputs: the same contraction with v_mfma_f32_16x16x4_f32, whose K-step is 4 consecutive pixels (lane ->
// row l%16, pixel l/16).  Operands are single dwords, so a tap is any element shift and nothing has to be cut;
// staging moves items of VEC adjacent pixels of a row (4 when W is a multiple of 4, else 2 or 1), at most
// kF32Items per thread and tensor, which wait in registers while the previous chunk is computed.
constexpr int kF32Items = 18;     // staging items per thread, tensor and chunk
constexpr int kGuardF = 4;       // zero floats in front of each X channel row
constexpr int kRowsThreads = 512;
constexpr int kRowsBatches = 2;   // staging batches (of 28 floats per thread and tensor) a chunk may need   // staging items per thread and tensor of the kernel for windows with a row extent

template <int KH, int KW, int CT, int VEC>
__global__ __launch_bounds__(256) void dw_mfma_f32(const DwParams p, const float* __restrict__ Gt,
                                                   const float* __restrict__ Xt, float* __restrict__ partial) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* gl = reinterpret_cast<float*>(smem);                   // [64][CPg]
  float* xl = reinterpret_cast<float*>(smem + p.lds_x_off);     // [32*CT][CPp], data starts at kGuardF
  int* row_tab = reinterpret_cast<int*>(smem + p.lds_tab_off);  // [2][n_xrows]
  constexpr int CX = 32 * CT, T = KH * KW;

  const int tid = threadIdx.x, lane = tid & 63;
  const int widx = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wo = widx >> 1, wc = widx & 1;
  int bid = blockIdx.x;
  const int split = bid % p.n_splits; bid /= p.n_splits;
  const int cb = bid % p.n_cblk; bid /= p.n_cblk;
  const int ob = bid % p.n_oblk;
  const int g = bid / p.n_oblk;
  const int chunk_begin = split * p.chunks_per_split;
  const int chunk_end = min(p.n_chunks, chunk_begin + p.chunks_per_split);
  {
    uint4* z = reinterpret_cast<uint4*>(smem);
    const int n16 = p.lds_tab_off >> 4;
    for (int i = tid; i < n16; i += 256) z[i] = make_uint4(0, 0, 0, 0);
  }
  const int o_lim = p.Og - ob * 64, c_lim = min(p.Cg - cb * CX, CX);
  const float* Gg = Gt + (int64_t)(g * p.Og + ob * 64) * p.plane;
  const float* Xg = Xt + (int64_t)(g * p.Cg + cb * CX) * p.plane;

  floatx4 acc[2][CT][T];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < CT; ++b)
#pragma unroll
      for (int t = 0; t < T; ++t) acc[a][b][t] = floatx4{0.f, 0.f, 0.f, 0.f};
  int a_base[2], b_base[CT];     // element indices
#pragma unroll
  for (int a = 0; a < 2; ++a) a_base[a] = ((2 * wo + a) * 16 + (lane & 15)) * p.CPg + (lane >> 4);
#pragma unroll
  for (int b = 0; b < CT; ++b) b_base[b] = ((CT * wc + b) * 16 + (lane & 15)) * p.CPp + (lane >> 4) + kGuardF - p.pw;

  // ---- staging items of this thread (the same for every chunk): VEC pixels of (channel, row)
  typedef float vec_t __attribute__((ext_vector_type(VEC == 1 ? 2 : VEC), aligned(4)));
  int it_off[kF32Items], it_r[kF32Items], it_lo[kF32Items], it_lg[kF32Items];
  {
    const int WV = p.W / VEC;                        // items per row
#pragma unroll
    for (int k = 0; k < kF32Items; ++k) {
      const int idx = tid + k * 256;
      const int ch = __umulhi((uint32_t)idx, p.magic_rw2);
      const int rem = idx - ch * (p.n_xrows * WV);
      const int r = p.magic_w2 ? __umulhi((uint32_t)rem, p.magic_w2) : rem;   // (one item per row: no division)
      const int j = (rem - r * WV) * VEC;
      const bool used = idx < p.items;
      it_off[k] = ch * p.plane + j;
      // bit 30 / 29: this channel exists in G / in X
      it_r[k] = used ? (r | (ch < o_lim ? (1 << 30) : 0) | (ch < c_lim ? (1 << 29) : 0)) : -1;
      it_lo[k] = (used && ch < CX) ? ch * p.CPp + r * p.pitch + j + kGuardF : -1;
      it_lg[k] = (used && r < p.TRK) ? ch * p.CPg + r * p.pitch + j : -1;
    }
  }
  float gr[kF32Items][VEC], xr[kF32Items][VEC];
  // source rows of chunk q: tab[r] = G row offset, tab[n_xrows + r] = X row offset (-1: none, zeros)
  auto rows_of = [&](int q, int tab) {     // tab: offset of the table inside row_tab (an index, so that LDS stays LDS)
    if (tid < p.n_xrows) {
      int go = -1, xo = -1;
      if (KH == 1) {
        const int rho = q * p.TRK + tid;
        if (rho < p.rows_total) {
          const int n = rho / p.H, h = rho - n * p.H;
          const int r = p.h_wrap ? (h + p.h_shift + p.h_shift_g * g) % p.H : h;
          go = n * p.gs_n + h * p.W;
          xo = n * p.xs_n + r * p.W;
        }
      } else {
        const int n = q / p.cpi, h0 = (q - n * p.cpi) * p.TRK;
        const int rows = min(p.TRK, p.H - h0);
        if (tid < rows) go = n * p.gs_n + (h0 + tid) * p.W;
        const int hx = h0 - p.ph + tid;
        if (tid < rows + KH - 1 && hx >= 0 && hx < p.H) xo = n * p.xs_n + hx * p.W;
      }
      row_tab[tab + tid] = go;
      row_tab[tab + p.n_xrows + tid] = xo;
    }
  };
  // global -> registers.  Every item is loaded unconditionally (items without a source read the block's first
  // elements) so that the requests go out back to back; what has no source is zeroed on the way to LDS.
  uint32_t g_ok = 0, x_ok = 0;           // bit k: item k of the chunk in flight has a source in G / in X
  auto load = [&](int tab) {
    g_ok = 0; x_ok = 0;
#pragma unroll
    for (int k = 0; k < kF32Items; ++k) {
      const int r = it_r[k] >= 0 ? (it_r[k] & 0xffff) : 0;
      const int go = row_tab[tab + r], xo = row_tab[tab + p.n_xrows + r];
      const bool gv = it_r[k] >= 0 && go >= 0 && (it_r[k] >> 30);
      const bool xv = it_r[k] >= 0 && xo >= 0 && ((it_r[k] >> 29) & 1);
      g_ok |= gv ? (1u << k) : 0u;
      x_ok |= xv ? (1u << k) : 0u;
      const float* gs = Gg + (gv ? go + it_off[k] : 0);
      const float* xs = Xg + (xv ? xo + it_off[k] : 0);
      if constexpr (VEC == 1) {
        gr[k][0] = *gs;
        xr[k][0] = *xs;
      } else {
        const vec_t a = *reinterpret_cast<const vec_t*>(gs);
        const vec_t b = *reinterpret_cast<const vec_t*>(xs);
#pragma unroll
        for (int e = 0; e < VEC; ++e) { gr[k][e] = a[e]; xr[k][e] = b[e]; }
      }
    }
  };
  auto store = [&]() {                   // registers -> LDS
#pragma unroll
    for (int k = 0; k < kF32Items; ++k) {
      if (it_lg[k] >= 0)
#pragma unroll
        for (int e = 0; e < VEC; ++e) gl[it_lg[k] + e] = ((g_ok >> k) & 1) ? gr[k][e] : 0.f;
      if (it_lo[k] >= 0)
#pragma unroll
        for (int e = 0; e < VEC; ++e) xl[it_lo[k] + e] = ((x_ok >> k) & 1) ? xr[k][e] : 0.f;
    }
  };

  // The next chunk travels global -> registers while the current one is computed out of LDS.
  const int tab[2] = {0, 2 * p.n_xrows};
  if (chunk_begin < chunk_end) {
    rows_of(chunk_begin, tab[0]);
    __syncthreads();                     // (also: the zero fill is complete)
    load(tab[0]);
  }
  for (int q = chunk_begin; q < chunk_end; ++q) {
    const bool more = q + 1 < chunk_end;
    const int next = ((q - chunk_begin + 1) & 1) ? tab[1] : tab[0];
    __syncthreads();                     // the previous chunk is fully consumed
    store();
    if (more) rows_of(q + 1, next);
    __syncthreads();
    if (more) load(next);
    dw_f32_chunk<KH, KW, CT>(p, gl, xl, a_base, b_base, acc);
  }
  dw_finish<KH, KW, CT>(p, partial, g, ob, cb, split, widx, lane, acc);
}

// fp32, windows with a row extent (KH = 3).  A chunk is TRK rows of ONE image, so the source of staged row r is
// row h0 + r of G and row h0 - 1 + r of X: one uniform base per chunk and tensor plus an offset that depends only on
// the item; nothing is looked up, and every load is a uniform base plus a 32-bit lane offset.
//
// Eight waves in two halves that trade places: while one half (4 waves, one per SIMD, each with its own part of the
// output tile) multiplies the chunk that lies in one LDS buffer, the other half fetches the next chunk from memory
// and lays it out in the second buffer; after one barrier the halves swap roles.  So each half computes every other
// chunk of the workgroup's share and stages the chunks it will compute itself; the matrix pipes always have a wave
// that issues MFMAs, and the memory round trips, the address arithmetic and the LDS writes of the staging all run
// beside them.  The sums of the two halves meet in LDS at the end.
// Staging goes in batches of up to 28 floats per thread and tensor: items of adjacent pixels of a row (a whole row of
// 7 or 14 pixels, else 4, 2 or 1 pixels), G (64 channels x TRK rows) and X (32*CT channels x TRK + 2 rows) together.  Rows that a chunk does not have (the halo above the
// first and below the last row of an image, the missing rows of an image's last chunk) are loaded from a safe
// address and written as zeros; items beyond the list or the group's channels go to 4 KB of LDS nobody reads.
template <int KW, int CT, int MODE>
__global__ __launch_bounds__(kRowsThreads) void dw_rows_f32(const DwParams p, const float* __restrict__ Gt,
                                                            const float* __restrict__ Xt, float* __restrict__ partial) {
  constexpr int KH = 3, CX = 32 * CT, T = KH * KW;
  // A staging item is MODE adjacent pixels of one staged row: 4, 2 or 1 (what the width divides by), or a whole row
  // of 7 or 14 pixels, moved as pieces of 4, 2 and 1.
  constexpr int FL = MODE;                                          // floats per item
  constexpr int NB = MODE == 7 ? 4 : MODE == 14 ? 2 : 7;            // items per thread and batch
  constexpr int NI = NB * kRowsBatches;                             // items per thread and chunk at most
  extern __shared__ __align__(16) unsigned char smem[];
  const uint32_t dump = (uint32_t)p.lds_tab_off;                // behind the two buffers

  const int tid = threadIdx.x, lane = tid & 63, htid = tid & 255;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int widx = wave & 3, half = wave >> 2;
  const int wo = widx >> 1, wc = widx & 1;
  int bid = blockIdx.x;
  const int split = bid % p.n_splits; bid /= p.n_splits;
  const int cb = bid % p.n_cblk; bid /= p.n_cblk;
  const int ob = bid % p.n_oblk;
  const int g = bid / p.n_oblk;
  const int chunk_begin = split * p.chunks_per_split;
  const int chunk_end = min(p.n_chunks, chunk_begin + p.chunks_per_split);
  {
    uint4* z = reinterpret_cast<uint4*>(smem);
    const int n16 = p.lds_tab_off >> 4;
    for (int i = tid; i < n16; i += kRowsThreads) z[i] = make_uint4(0, 0, 0, 0);
  }
  const int o_lim = p.Og - ob * 64, c_lim = min(p.Cg - cb * CX, CX);
  const float* Gg = Gt + (int64_t)(g * p.Og + ob * 64) * p.plane;
  const float* Xg = Xt + (int64_t)(g * p.Cg + cb * CX) * p.plane;

  floatx4 acc[2][CT][T];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < CT; ++b)
#pragma unroll
      for (int t = 0; t < T; ++t) acc[a][b][t] = floatx4{0.f, 0.f, 0.f, 0.f};
  int a_base[2], b_base[CT];     // element indices inside a buffer's G and X tile
#pragma unroll
  for (int a = 0; a < 2; ++a) a_base[a] = ((2 * wo + a) * 16 + (lane & 15)) * p.CPg + (lane >> 4);
#pragma unroll
  for (int b = 0; b < CT; ++b) b_base[b] = ((CT * wc + b) * 16 + (lane & 15)) * p.CPp + (lane >> 4) + kGuardF - p.pw;

  // ---- this thread's staging items, worked out once.  256 threads of a half share a tensor's channels evenly
  // (4 threads per G channel, 256 / CX per X channel); a thread takes every 4th (8th) item of its channel.  Per
  // item: the byte offset from the chunk's first source row, and the LDS byte offset inside a buffer with the staged
  // row in the top byte (row 255: never).
  uint32_t g_off[NI], g_put[NI], x_off[NI], x_put[NI];
  {
    const int WR = p.W / FL;                     // items per row
    auto plan_items = [&](uint32_t (&off)[NI], uint32_t (&put)[NI], int tpc_log2, int rows_staged, int ch_lim,
                          int ch_pitch, int lds_first, uint32_t safe) {
      const int ch = htid >> tpc_log2, sub = htid & ((1 << tpc_log2) - 1);
#pragma unroll
      for (int k = 0; k < NI; ++k) {
        const int i = sub + (k << tpc_log2);
        const int r = p.magic_w2 ? (int)__umulhi((uint32_t)i, p.magic_w2) : i;
        const int j = (i - r * WR) * FL;
        const bool exists = r < rows_staged && ch < ch_lim;
        off[k] = exists ? (uint32_t)(ch * p.plane + r * p.W + j) * 4 : safe;
        // (items that never carry data write to a spare area behind the buffers, each lane to its own 64 bytes)
        put[k] = exists ? ((uint32_t)(lds_first + ch * ch_pitch + r * p.pitch + j) * 4) | ((uint32_t)r << 24)
                        : (dump + (uint32_t)lane * 64) | (255u << 24);
      }
    };
    plan_items(g_off, g_put, 2, p.TRK, o_lim, p.CPg, 0, 0u);
    plan_items(x_off, x_put, CT == 1 ? 3 : 2, p.n_xrows, c_lim, p.CPp, kGuardF + (p.lds_x_off >> 2), (uint32_t)p.W * 4);
  }
  // Pieces of an item: float offset and width.  Source rows are only element-aligned; in LDS a row of 7 starts on a
  // 32-byte boundary (pitch 8), every other layout is element-aligned as well.
  typedef float f4_t __attribute__((ext_vector_type(4), aligned(4)));
  typedef float f2_t __attribute__((ext_vector_type(2), aligned(4)));
  typedef float f4a_t __attribute__((ext_vector_type(4), aligned(16)));
  typedef float f2a_t __attribute__((ext_vector_type(2), aligned(8)));
  auto load_item = [&](float (&v)[FL], const char* src) {
    const float* f = reinterpret_cast<const float*>(src);
    int o = 0;
#pragma unroll
    for (; o + 4 <= FL; o += 4) { const f4_t t = *reinterpret_cast<const f4_t*>(f + o); v[o] = t[0]; v[o + 1] = t[1]; v[o + 2] = t[2]; v[o + 3] = t[3]; }
    if constexpr (FL % 4 >= 2) { const f2_t t = *reinterpret_cast<const f2_t*>(f + o); v[o] = t[0]; v[o + 1] = t[1]; o += 2; }
    if constexpr (FL % 2 == 1) v[o] = f[o];
  };
  auto store_item = [&](const float (&v)[FL], unsigned char* dst) {
    float* f = reinterpret_cast<float*>(dst);
    int o = 0;
#pragma unroll
    for (; o + 4 <= FL; o += 4) {
      if constexpr (MODE == 7) *reinterpret_cast<f4a_t*>(f + o) = f4a_t{v[o], v[o + 1], v[o + 2], v[o + 3]};
      else *reinterpret_cast<f4_t*>(f + o) = f4_t{v[o], v[o + 1], v[o + 2], v[o + 3]};
    }
    if constexpr (FL % 4 >= 2) {
      if constexpr (MODE == 7) *reinterpret_cast<f2a_t*>(f + o) = f2a_t{v[o], v[o + 1]};
      else *reinterpret_cast<f2_t*>(f + o) = f2_t{v[o], v[o + 1]};
      o += 2;
    }
    if constexpr (FL % 2 == 1) f[o] = v[o];
  };
  // One batch of one tensor: up to NB items, requested back to back; staged rows [r_lo, r_hi) exist in this chunk.
  struct Batch { float v[NB][FL]; };
  auto fetch = [&](Batch& bt, const char* src_base, const uint32_t* off, const uint32_t* put, int count, uint32_t safe,
                   int r_lo, int r_hi) {
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      if (k >= count) break;
      const bool ok = ((put[k] >> 24) - (uint32_t)r_lo) < (uint32_t)(r_hi - r_lo);
      load_item(bt.v[k], src_base + (ok ? off[k] : safe));
    }
  };
  auto put_batch = [&](Batch& bt, uint32_t buf, const uint32_t* put, int count, int r_lo, int r_hi) {
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      if (k >= count) break;
      const bool ok = ((put[k] >> 24) - (uint32_t)r_lo) < (uint32_t)(r_hi - r_lo);
      const bool never = (put[k] >> 24) == 255u;
#pragma unroll
      for (int e = 0; e < FL; ++e) bt.v[k][e] = ok ? bt.v[k][e] : 0.f;
      store_item(bt.v[k], smem + (put[k] & 0xffffffu) + (never ? 0u : buf));
    }
  };
  // Stages chunk q (rows [h0, h0 + rows) of image n) into the buffer at byte offset `buf`; run by the 256 threads of
  // one half.  The batches of G and X are requested together, then written.
  auto stage = [&](int q, uint32_t buf) {
    const int n = p.magic_cpi ? (int)__umulhi((uint32_t)q, p.magic_cpi) : q;
    const int h0 = (q - n * p.cpi) * p.TRK;
    const int rows = min(p.TRK, p.H - h0);
    const char* gb = reinterpret_cast<const char*>(Gg) + ((int64_t)n * p.gs_n + (int64_t)h0 * p.W) * 4;
    // (one row above the chunk; when the chunk starts an image that row is not read: staged row 0 does not exist then
    // and the safe offset points at the chunk's first row)
    const char* xb = reinterpret_cast<const char*>(Xg) + ((int64_t)n * p.xs_n + (int64_t)(h0 - 1) * p.W) * 4;
    const int x_lo = h0 == 0 ? 1 : 0, x_hi = min(rows + 2, p.H - h0 + 1);
#pragma unroll
    for (int b = 0; b < NI / NB; ++b) {
      const int ng = p.ni_g - b * NB, nx = p.ni_x - b * NB;       // (uniform) items of this batch
      if (ng <= 0 && nx <= 0) break;
      Batch bg, bx;
      fetch(bg, gb, g_off + b * NB, g_put + b * NB, ng, 0u, 0, rows);
      fetch(bx, xb, x_off + b * NB, x_put + b * NB, nx, (uint32_t)p.W * 4, x_lo, x_hi);
      put_batch(bg, buf, g_put + b * NB, ng, 0, rows);
      put_batch(bx, buf, x_put + b * NB, nx, x_lo, x_hi);
    }
  };

  __syncthreads();                                   // LDS is zeroed
  if (half == 0 && chunk_begin < chunk_end) stage(chunk_begin, 0u);
  __syncthreads();
  for (int q = chunk_begin; q < chunk_end; ++q) {
    const int par = (q - chunk_begin) & 1;
    if (par == half) {
      const unsigned char* cur = smem + par * p.lds_buf;
      dw_f32_chunk<KH, KW, CT>(p, reinterpret_cast<const float*>(cur), reinterpret_cast<const float*>(cur + p.lds_x_off),
                               a_base, b_base, acc);
    } else if (q + 1 < chunk_end) {
      stage(q + 1, (uint32_t)((par ^ 1) * p.lds_buf));
    }
    __syncthreads();
  }
  // the sums of the two halves meet in LDS: the upper waves leave theirs there, the lower ones add them
  floatx4* red = reinterpret_cast<floatx4*>(smem) + (widx * 2 * CT * T) * 64 + lane;
  if (half) {
#pragma unroll
    for (int ao = 0; ao < 2; ++ao)
#pragma unroll
      for (int i = 0; i < CT; ++i)
#pragma unroll
        for (int t = 0; t < T; ++t) red[((ao * CT + i) * T + t) * 64] = acc[ao][i][t];
  }
  __syncthreads();
  if (half) return;
#pragma unroll
  for (int ao = 0; ao < 2; ++ao)
#pragma unroll
    for (int i = 0; i < CT; ++i)
#pragma unroll
      for (int t = 0; t < T; ++t) acc[ao][i][t] += red[((ao * CT + i) * T + t) * 64];
  dw_finish<KH, KW, CT>(p, partial, g, ob, cb, split, widx, lane, acc);
}

// The same design for bf16 inputs (v_mfma_f32_16x16x32_bf16, k-steps of 32 pixels, taps cut out of aligned 16-byte
// reads): two halves of four waves trade places between multiplying the chunk in one LDS buffer and staging the next
// chunk into the other.  A staging item is MODE adjacent pixels of one staged row: 4 (8 bytes), 2 or 1, or a whole row
// of 7 or 14 pixels; rows in LDS start on 16-byte boundaries (the pitch is a multiple of 8 elements), source rows are
// aligned to an item's size except the whole-row items, which are read as unaligned pieces.
template <int KW, int CT, int MODE>
__global__ __launch_bounds__(kRowsThreads) void dw_rows_bf16(const DwParams p, const uint16_t* __restrict__ Gt,
                                                             const uint16_t* __restrict__ Xt, float* __restrict__ partial) {
  constexpr int KH = 3, CX = 32 * CT, T = KH * KW;
  constexpr int NB = MODE == 7 ? 4 : MODE == 14 ? 2 : 7;            // items per thread and batch
  constexpr int NI = NB * kRowsBatches;                             // items per thread and chunk at most                             // items per thread and chunk at most
  constexpr int DW = (MODE + 1) / 2;                                // dwords that hold an item
  extern __shared__ __align__(16) unsigned char smem[];
  const uint32_t dump = (uint32_t)p.lds_tab_off;                // behind the two buffers

  const int tid = threadIdx.x, lane = tid & 63, htid = tid & 255;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int widx = wave & 3, half = wave >> 2;
  const int wo = widx >> 1, wc = widx & 1;
  int bid = blockIdx.x;
  const int split = bid % p.n_splits; bid /= p.n_splits;
  const int cb = bid % p.n_cblk; bid /= p.n_cblk;
  const int ob = bid % p.n_oblk;
  const int g = bid / p.n_oblk;
  const int chunk_begin = split * p.chunks_per_split;
  const int chunk_end = min(p.n_chunks, chunk_begin + p.chunks_per_split);
  {
    uint4* z = reinterpret_cast<uint4*>(smem);
    const int n16 = p.lds_tab_off >> 4;
    for (int i = tid; i < n16; i += kRowsThreads) z[i] = make_uint4(0, 0, 0, 0);
  }
  const int o_lim = p.Og - ob * 64, c_lim = min(p.Cg - cb * CX, CX);
  const uint16_t* Gg = Gt + (int64_t)(g * p.Og + ob * 64) * p.plane;
  const uint16_t* Xg = Xt + (int64_t)(g * p.Cg + cb * CX) * p.plane;

  floatx4 acc[2][CT][T];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < CT; ++b)
#pragma unroll
      for (int t = 0; t < T; ++t) acc[a][b][t] = floatx4{0.f, 0.f, 0.f, 0.f};
  int a_base[2], b_base[CT];     // element indices inside a buffer's G and X tile
#pragma unroll
  for (int a = 0; a < 2; ++a) a_base[a] = ((2 * wo + a) * 16 + (lane & 15)) * p.CPg + (lane >> 4) * 8;
#pragma unroll
  for (int b = 0; b < CT; ++b) b_base[b] = ((CT * wc + b) * 16 + (lane & 15)) * p.CPp + (lane >> 4) * 8 + kGuard - 8;

  // ---- this thread's staging items, worked out once (4 threads per G channel, 256 / CX per X channel; a thread takes
  // every 4th (8th) item of its channel): byte offset from the chunk's first source row, and the LDS byte offset
  // inside a buffer with the staged row in the top byte (row 255: never)
  uint32_t g_off[NI], g_put[NI], x_off[NI], x_put[NI];
  {
    const int WR = p.W / MODE;                   // items per row
    // With several whole images per chunk, image i of the chunk has H + 2 staged rows of its own: row l holds G row l
    // (the last two stay zero) and X row l - 1 (zero outside the image).
    const int per = p.H + 2;
    auto plan_items = [&](uint32_t (&off)[NI], uint32_t (&put)[NI], int tpc_log2, int rows_staged, int ch_lim,
                          int ch_pitch, int lds_first, uint32_t safe, int image_stride, int l_lo, int l_hi) {
      const int ch = htid >> tpc_log2, sub = htid & ((1 << tpc_log2) - 1);
#pragma unroll
      for (int k = 0; k < NI; ++k) {
        const int i = sub + (k << tpc_log2);
        const int r = p.magic_w2 ? (int)__umulhi((uint32_t)i, p.magic_w2) : i;
        const int j = (i - r * WR) * MODE;
        const int img = p.ipc > 1 ? r / per : 0, l = r - img * per;
        const bool exists = r < rows_staged && ch < ch_lim && (p.ipc == 1 || (l >= l_lo && l < l_hi));
        off[k] = exists ? (uint32_t)(img * image_stride + ch * p.plane + l * p.W + j) * 2 : safe;
        put[k] = exists ? ((uint32_t)(lds_first + ch * ch_pitch + r * p.pitch + j) * 2) | ((uint32_t)r << 24)
                        : (dump + (uint32_t)lane * 64) | (255u << 24);
      }
    };
    plan_items(g_off, g_put, 2, p.ipc > 1 ? p.n_xrows : p.TRK, o_lim, p.CPg, 0, 0u, p.gs_n, 0, p.H);
    plan_items(x_off, x_put, CT == 1 ? 3 : 2, p.n_xrows, c_lim, p.CPp, kGuard + (p.lds_x_off >> 1), (uint32_t)p.W * 2,
               p.xs_n, 1, p.H + 1);
  }
  typedef uint32_t u4_t __attribute__((ext_vector_type(4), aligned(4)));
  typedef uint32_t u2_t __attribute__((ext_vector_type(2), aligned(4)));
  typedef uint32_t u2h_t __attribute__((ext_vector_type(2), aligned(2)));
  typedef uint32_t u1h_t __attribute__((aligned(2)));
  auto load_item = [&](uint32_t (&v)[DW], const char* src) {
    if constexpr (MODE == 4) {
      const uint2 t = *reinterpret_cast<const uint2*>(src);
      v[0] = t.x; v[1] = t.y;
    } else if constexpr (MODE == 2) {
      v[0] = *reinterpret_cast<const uint32_t*>(src);
    } else if constexpr (MODE == 1) {
      v[0] = *reinterpret_cast<const uint16_t*>(src);
    } else if constexpr (MODE == 14) {      // 28 bytes, dword-aligned
      const u4_t a = *reinterpret_cast<const u4_t*>(src);
      const u2_t b = *reinterpret_cast<const u2_t*>(src + 16);
      v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3]; v[4] = b[0]; v[5] = b[1];
      v[6] = *reinterpret_cast<const uint32_t*>(src + 24);
    } else {                                 // 14 bytes, element-aligned
      const u2h_t a = *reinterpret_cast<const u2h_t*>(src);
      v[0] = a[0]; v[1] = a[1];
      v[2] = *reinterpret_cast<const u1h_t*>(src + 8);
      v[3] = *reinterpret_cast<const uint16_t*>(src + 12);
    }
  };
  auto store_item = [&](const uint32_t (&v)[DW], unsigned char* dst) {     // (LDS rows start on 16-byte boundaries)
    if constexpr (MODE == 4) {
      *reinterpret_cast<uint2*>(dst) = make_uint2(v[0], v[1]);
    } else if constexpr (MODE == 2) {
      *reinterpret_cast<uint32_t*>(dst) = v[0];
    } else if constexpr (MODE == 1) {
      *reinterpret_cast<uint16_t*>(dst) = (uint16_t)v[0];
    } else if constexpr (MODE == 14) {
      *reinterpret_cast<uint4*>(dst) = make_uint4(v[0], v[1], v[2], v[3]);
      *reinterpret_cast<uint2*>(dst + 16) = make_uint2(v[4], v[5]);
      *reinterpret_cast<uint32_t*>(dst + 24) = v[6];
    } else {
      *reinterpret_cast<uint2*>(dst) = make_uint2(v[0], v[1]);
      *reinterpret_cast<uint32_t*>(dst + 8) = v[2];
      *reinterpret_cast<uint16_t*>(dst + 12) = (uint16_t)v[3];
    }
  };
  struct Batch { uint32_t v[NB][DW]; };
  auto fetch = [&](Batch& bt, const char* src_base, const uint32_t* off, const uint32_t* put, int count, uint32_t safe,
                   int r_lo, int r_hi) {
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      if (k >= count) break;
      const bool ok = ((put[k] >> 24) - (uint32_t)r_lo) < (uint32_t)(r_hi - r_lo);
      load_item(bt.v[k], src_base + (ok ? off[k] : safe));
    }
  };
  auto put_batch = [&](Batch& bt, uint32_t buf, const uint32_t* put, int count, int r_lo, int r_hi) {
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      if (k >= count) break;
      const bool ok = ((put[k] >> 24) - (uint32_t)r_lo) < (uint32_t)(r_hi - r_lo);
      const bool never = (put[k] >> 24) == 255u;
#pragma unroll
      for (int e = 0; e < DW; ++e) bt.v[k][e] = ok ? bt.v[k][e] : 0u;
      store_item(bt.v[k], smem + (put[k] & 0xffffffu) + (never ? 0u : buf));
    }
  };
  auto stage = [&](int q, uint32_t buf) {
    int n = p.magic_cpi ? (int)__umulhi((uint32_t)q, p.magic_cpi) : q;
    int h0 = (q - n * p.cpi) * p.TRK;
    int rows = min(p.TRK, p.H - h0);
    int x_lo = h0 == 0 ? 1 : 0, x_hi = min(rows + 2, p.H - h0 + 1);
    if (p.ipc > 1) {                // whole images q*ipc ..: every staged row of an image that the batch has exists
      n = q * p.ipc; h0 = 0;
      rows = min(p.ipc, p.n_images - n) * (p.H + 2);
      x_lo = 0; x_hi = rows;
    }
    const char* gb = reinterpret_cast<const char*>(Gg) + ((int64_t)n * p.gs_n + (int64_t)h0 * p.W) * 2;
    // (one row above the chunk; when the chunk starts an image that row is not read: staged row 0 does not exist then
    // and the safe offset points at the chunk's first row)
    const char* xb = reinterpret_cast<const char*>(Xg) + ((int64_t)n * p.xs_n + (int64_t)(h0 - 1) * p.W) * 2;
#pragma unroll
    for (int b = 0; b < NI / NB; ++b) {
      const int ng = p.ni_g - b * NB, nx = p.ni_x - b * NB;       // (uniform) items of this batch
      if (ng <= 0 && nx <= 0) break;
      Batch bg, bx;
      fetch(bg, gb, g_off + b * NB, g_put + b * NB, ng, 0u, 0, rows);
      fetch(bx, xb, x_off + b * NB, x_put + b * NB, nx, (uint32_t)p.W * 2, x_lo, x_hi);
      put_batch(bg, buf, g_put + b * NB, ng, 0, rows);
      put_batch(bx, buf, x_put + b * NB, nx, x_lo, x_hi);
    }
  };

  __syncthreads();                                   // LDS is zeroed
  if (half == 0 && chunk_begin < chunk_end) stage(chunk_begin, 0u);
  __syncthreads();
  for (int q = chunk_begin; q < chunk_end; ++q) {
    const int par = (q - chunk_begin) & 1;
    if (par == half) {
      const unsigned char* cur = smem + par * p.lds_buf;
      dw_bf16_chunk<KH, KW, CT>(p, reinterpret_cast<const uint16_t*>(cur),
                                reinterpret_cast<const uint16_t*>(cur + p.lds_x_off), a_base, b_base, acc);
    } else if (q + 1 < chunk_end) {
      stage(q + 1, (uint32_t)((par ^ 1) * p.lds_buf));
    }
    __syncthreads();
  }
  // the sums of the two halves meet in LDS: the upper waves leave theirs there, the lower ones add them
  floatx4* red = reinterpret_cast<floatx4*>(smem) + (widx * 2 * CT * T) * 64 + lane;
  if (half) {
#pragma unroll
    for (int ao = 0; ao < 2; ++ao)
#pragma unroll
      for (int i = 0; i < CT; ++i)
#pragma unroll
        for (int t = 0; t < T; ++t) red[((ao * CT + i) * T + t) * 64] = acc[ao][i][t];
  }
  __syncthreads();
  if (half) return;
#pragma unroll
  for (int ao = 0; ao < 2; ++ao)
#pragma unroll
    for (int i = 0; i < CT; ++i)
#pragma unroll
      for (int t = 0; t < T; ++t) acc[ao][i][t] += red[((ao * CT + i) * T + t) * 64];
  dw_finish<KH, KW, CT>(p, partial, g, ob, cb, split, widx, lane, acc);
}

// Adds the split partials kept in the accumulator layout of the contraction kernels and writes the sums into dW;
// the variant for few splits of a large dW.  A block owns one 16 (o) x 16 (c) tile with all its T taps: T
// consecutive slots of 64 quadruples, slot = ((wave*2 + ao)*ct + i)*T + t naming the o-tile 2*(wave>>1) + ao and the
// c-tile ct*(wave&1) + i; lane l of a quadruple holds rows 4*(l>>4) .. +3 (o) of column l&15 (c).  Wave j adds the
// splits, in order, for taps j, j+4, ...; then the threads walk the tile in (o, c, tap) order, which is contiguous in
// dW for the usual weight layouts, so dW is written in whole lines.
constexpr int kMaxTaps = 9;
__global__ __launch_bounds__(256) void dw_reduce_tiles(const DwParams p, const float4* __restrict__ partial,
                                                       float* __restrict__ dW) {
  __shared__ float sums[kMaxTaps][64][4];
  const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int T = p.KH * p.KW;
  const int subs = p.slots / T;                    // 16x16 tiles per workgroup tile
  const int tile = blockIdx.x / subs, sub = blockIdx.x - tile * subs;
  const int64_t n4 = (int64_t)p.n_tiles * p.slots * 64;
  for (int t = grp; t < T; t += 4) {
    const int64_t e = ((int64_t)tile * p.slots + sub * T + t) * 64 + lane;
    float4 s = partial[e];
    for (int k = 1; k < p.n_splits; ++k) {
      const float4 v = partial[(int64_t)k * n4 + e];
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    *reinterpret_cast<float4*>(sums[t][lane]) = s;
  }
  __syncthreads();
  int q = tile;
  const int cb = q % p.n_cblk; q /= p.n_cblk;
  const int ob = q % p.n_oblk;
  const int g = q / p.n_oblk;
  const int i = sub % p.ct, ao = (sub / p.ct) & 1, wave = sub / (p.ct * 2);
  const int c0 = cb * 32 * p.ct + (p.ct * (wave & 1) + i) * 16;
  // thread = (row ol, 16 threads per row); a row is 16*T consecutive (c, tap) pairs
  const int ol = threadIdx.x >> 4, o = ob * 64 + (2 * (wave >> 1) + ao) * 16 + ol;
  if (o >= p.Og) return;
  const uint32_t inv_t = (65536u + T - 1) / T;      // rem / T for rem < 16 * kMaxTaps
  const int64_t row = (int64_t)g * p.ws_g + (int64_t)o * p.ws_o;
  for (int rem = threadIdx.x & 15; rem < 16 * T; rem += 16) {
    const int cl = (int)(((uint32_t)rem * inv_t) >> 16), t = rem - cl * T;
    const int c = c0 + cl;
    if (c >= p.Cg) continue;
    const int kh = t / p.KW;
    dW[row + (int64_t)c * p.ws_c + kh * p.ws_kh + (t - kh * p.KW) * p.ws_kw] = sums[t][(ol >> 2) * 16 + cl][ol & 3];
  }
}

// The same sums for many splits and few tiles: a block owns one slot (64 quadruples, one tap of a 16x16 tile), which
// keeps enough blocks in flight when dW is small; the stores are scattered, which does not matter at that size.
__global__ __launch_bounds__(256) void dw_reduce_slots(const DwParams p, const float4* __restrict__ partial,
                                                       float* __restrict__ dW) {
  __shared__ float4 sums[4][64];
  const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int64_t n4 = (int64_t)p.n_tiles * p.slots * 64;
  const int64_t e = (int64_t)blockIdx.x * 64 + lane;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
  for (int k = grp; k < p.n_splits; k += 4) {
    const float4 v = partial[(int64_t)k * n4 + e];
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  sums[grp][lane] = s;
  __syncthreads();
  if (grp != 0) return;
  const float4 a = sums[0][lane], b = sums[1][lane], c4 = sums[2][lane], d = sums[3][lane];
  const float r[4] = {(a.x + b.x) + (c4.x + d.x), (a.y + b.y) + (c4.y + d.y), (a.z + b.z) + (c4.z + d.z),
                      (a.w + b.w) + (c4.w + d.w)};
  const int T = p.KH * p.KW;
  int q = blockIdx.x;
  const int slot = q % p.slots; q /= p.slots;
  const int cb = q % p.n_cblk; q /= p.n_cblk;
  const int ob = q % p.n_oblk;
  const int g = q / p.n_oblk;
  const int t = slot % T, sub = slot / T;
  const int i = sub % p.ct, ao = (sub / p.ct) & 1, wave = sub / (p.ct * 2);
  const int c = cb * 32 * p.ct + (p.ct * (wave & 1) + i) * 16 + (lane & 15);
  if (c >= p.Cg) return;
  const int64_t base = (int64_t)g * p.ws_g + (int64_t)c * p.ws_c + (t / p.KW) * p.ws_kh + (t % p.KW) * p.ws_kw;
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int o = ob * 64 + (2 * (wave >> 1) + ao) * 16 + 4 * (lane >> 4) + v;
    if (o < p.Og) dW[base + (int64_t)o * p.ws_o] = r[v];
  }
}

uint32_t magic_of(int d) { return (uint32_t)(((1ull << 32) + d - 1) / d); }

bool fill_dw(const syno_plan* plan, DwParams& p) {
  const ConvLike& c = plan->conv;
  p = DwParams{};
  p.G = c.G; p.Og = c.Og; p.Cg = c.Cg; p.H = c.Ho; p.W = c.Wo; p.KH = c.KH; p.KW = c.KW; p.ph = c.ph; p.pw = c.pw;
  p.rows_total = c.N * c.Ho;
  p.h_wrap = c.h_wrap; p.h_shift = c.h_shift; p.h_shift_g = c.h_shift_g;
  p.plane = c.Ho * c.Wo;
  p.gs_n = c.G * c.Og * p.plane; p.xs_n = c.G * c.Cg * p.plane;
  p.ws_g = c.ws_g; p.ws_o = c.ws_o; p.ws_c = c.ws_c; p.ws_kh = c.ws_kh; p.ws_kw = c.ws_kw;
  p.w_elems = (int32_t)plan->w_elems;
  p.pitch = (c.Wo + std::max(c.pw, c.KW - 1 - c.pw) + 1) & ~1;
  if (p.pitch == c.Wo) p.pitch += 2;                 // always at least one zero column
  if (c.KH > 1) p.pitch = (p.pitch + 7) & ~7;        // whole-row shifts stay 16-byte aligned
  const int cx = (c.KH * c.KW <= 3) ? 64 : 32;       // X channels per workgroup
  // rows per chunk: about 224 staged elements per channel, bounded by the per-thread item budget
  const int ep = (c.Wo % 4 == 0) ? 4 : (c.Wo % 2 == 0) ? 2 : 1;   // pixels per staging item
  const int W2 = c.Wo / ep, halo = c.KH - 1;                       // items per row
  if (ep == 4) p.pitch = (p.pitch + 3) & ~3;                      // 8-byte LDS writes
  if (c.KH == 3 && (c.Wo == 7 || c.Wo == 14)) {
    // windows with a row extent on narrow images (whole rows as staging items): the kernel whose wave halves alternate
    // between multiplying and staging.  Chunks as large as the per-thread item lists and two LDS buffers allow: rows
    // of one image, or several whole small images.  (Measured slower than the table kernel on 28- and 56-pixel rows,
    // whose 8-byte items it fetches four lanes to a channel: they stay there.)
    const int mode = (c.Wo == 7 || c.Wo == 14) ? c.Wo : ep;
    const int ni_cap = (mode == 7 ? 4 : mode == 14 ? 2 : 7) * kRowsBatches;
    const int wr = c.Wo / mode;
    auto skew = [](int v) { v = (v + 7) & ~7; return (v & 31) == 0 ? v + 8 : v; };
    auto cfg = [&](int t, int ipc, DwParams& o) {     // t rows of an image per chunk, or ipc whole images
      o = p;
      const int per = c.Ho + 2;
      o.ipc = ipc;
      o.n_xrows = ipc > 1 ? ipc * per : t + 2;
      o.TRK = ipc > 1 ? o.n_xrows - 2 : t;
      o.CP = (o.TRK * o.pitch + 31) & ~31;
      o.CPg = skew(o.CP + 8);
      o.CPp = skew(std::max(o.CP, o.n_xrows * o.pitch) + 2 * o.pitch + 48);
      o.ni_g = ((ipc > 1 ? o.n_xrows : t) * wr + 3) / 4;
      o.ni_x = (o.n_xrows * wr + 256 / cx - 1) / (256 / cx);
      o.lds_x_off = 64 * o.CPg * 2;
      o.lds_buf = o.lds_x_off + cx * o.CPp * 2;
      o.lds_tab_off = 2 * o.lds_buf;
      o.lds_bytes = std::max(o.lds_tab_off + 4096, 4 * 2 * (cx / 32) * c.KH * c.KW * 1024);
      return std::max(o.ni_g, o.ni_x) <= ni_cap && o.lds_bytes <= 160 * 1024 && o.n_xrows <= 254;
    };
    DwParams best;
    int t = c.Ho;
    while (t > 1 && !cfg(t, 1, best)) --t;
    if (!cfg(t, 1, best)) return false;
    if (t == c.Ho) {                 // whole images: as many per chunk as fit
      int m = 1;
      DwParams more;
      while (m < c.N && cfg(c.Ho, m + 1, more)) { best = more; ++m; }
      best.cpi = 1;
      best.n_chunks = (c.N + best.ipc - 1) / best.ipc;
    } else {
      best.cpi = (c.Ho + t - 1) / t;
      const int tb = (c.Ho + best.cpi - 1) / best.cpi;       // chunks of an image about equally long
      cfg(tb, 1, best);
      best.cpi = (c.Ho + tb - 1) / tb;
      best.n_chunks = c.N * best.cpi;
    }
    p = best;
    p.n_images = c.N;
    p.mode = mode;
    p.direct = 1;
    p.magic_w2 = magic_of(wr);
    p.magic_cpi = magic_of(p.cpi);
    p.n_oblk = (c.Og + 63) / 64;
    p.n_cblk = (c.Cg + cx - 1) / cx;
    const int tiles = c.G * p.n_oblk * p.n_cblk;
    p.n_tiles = tiles;
    p.ct = cx / 32;
    p.slots = 8 * p.ct * c.KH * c.KW;
    const int target = plan->opt.dw_workgroups > 0 ? plan->opt.dw_workgroups : 256;
    int splits = std::max(1, std::min(p.n_chunks, target / std::max(1, tiles)));
    while (splits > 1 && (int64_t)splits * tiles * p.slots * 1024 > (40ll << 20)) splits /= 2;
    p.chunks_per_split = (p.n_chunks + splits - 1) / splits;
    p.rows_per_split = p.chunks_per_split * p.TRK;
    p.n_splits = (p.n_chunks + p.chunks_per_split - 1) / p.chunks_per_split;
    return true;
  }
  int trk = std::max(1, 224 / p.pitch);
  if (c.KH > 1) trk = std::min(trk, c.Ho);
  while (trk > 1 && 64 * (trk + halo) * W2 > dw_items(ep) * 256) --trk;
  if (64 * (trk + halo) * W2 > dw_items(ep) * 256) return false;
  if (c.KH > 1) {
    p.cpi = (c.Ho + trk - 1) / trk;                   // chunks stay inside an image, all about equally long
    trk = (c.Ho + p.cpi - 1) / p.cpi;
    p.n_chunks = c.N * p.cpi;
  } else {
    trk = std::min(trk, p.rows_total);
    p.n_chunks = (p.rows_total + trk - 1) / trk;
  }
  p.TRK = trk;
  p.n_xrows = trk + halo;
  p.ipc = 1; p.n_images = c.N;
  if (c.KH > 1 && p.cpi == 1) {
    // whole small images: as many per chunk as the item budget and about 1024 staged elements per channel allow
    const int per = c.Ho + halo;
    int m = 1;
    while (m < c.N && 64 * (m + 1) * per * W2 <= dw_items(ep) * 256 && (m + 1) * per * p.pitch <= 1024) ++m;
    if (m > 1) {
      p.ipc = m;
      p.n_xrows = m * per;
      p.TRK = p.n_xrows - halo;
      p.n_chunks = (c.N + m - 1) / m;
    }
  }
  p.CP = (p.TRK * p.pitch + 31) & ~31;
  // LDS channel pitch: the last k-step reads up to CP + halo rows + 24 elements; guard in front, rows 16-byte
  // aligned and bank-skewed
  p.CPp = std::max(p.CP, p.n_xrows * p.pitch) + halo * p.pitch + 24;
  p.CPp = (p.CPp + 7) & ~7;
  if ((p.CPp & 31) == 0) p.CPp += 8;
  p.items = 64 * p.n_xrows * W2;
  p.magic_w2 = magic_of(W2);
  p.magic_rw2 = magic_of(p.n_xrows * W2);
  p.n_oblk = (c.Og + 63) / 64;
  p.n_cblk = (c.Cg + cx - 1) / cx;
  // split the chunks: aim at one workgroup per CU, keep the partials below ~32 MB
  const int tiles = c.G * p.n_oblk * p.n_cblk;
  p.n_tiles = tiles;
  p.ct = cx / 32;
  p.slots = 8 * p.ct * c.KH * c.KW;
  const int target = plan->opt.dw_workgroups > 0 ? plan->opt.dw_workgroups : 256;
  int splits = std::max(1, std::min(p.n_chunks, target / std::max(1, tiles)));
  while (splits > 1 && (int64_t)splits * tiles * p.slots * 1024 > (40ll << 20)) splits /= 2;
  p.chunks_per_split = (p.n_chunks + splits - 1) / splits;
  p.rows_per_split = p.chunks_per_split * p.TRK;
  p.n_splits = (p.n_chunks + p.chunks_per_split - 1) / p.chunks_per_split;
  p.lds_x_off = 64 * p.CPp * 2;
  p.lds_tab_off = p.lds_x_off + cx * p.CPp * 2;
  p.lds_bytes = p.lds_tab_off + ((2 * p.n_xrows * 4 + 15) & ~15);
  return p.lds_bytes <= 144 * 1024 && 64 * p.CPp < (1 << 20) && p.n_xrows < 1024 && p.n_xrows <= 256;
}

// fp32 configuration: element items, k-steps of 4 pixels, channel pitch = 4 * odd floats so that the 16 rows x 4
// pixels of a fragment read fall into 64 distinct banks.
bool fill_dw_f32_as(const syno_plan* plan, DwParams& p, bool direct) {
  const ConvLike& c = plan->conv;
  p = DwParams{};
  p.G = c.G; p.Og = c.Og; p.Cg = c.Cg; p.H = c.Ho; p.W = c.Wo; p.KH = c.KH; p.KW = c.KW; p.ph = c.ph; p.pw = c.pw;
  p.rows_total = c.N * c.Ho;
  p.h_wrap = c.h_wrap; p.h_shift = c.h_shift; p.h_shift_g = c.h_shift_g;
  p.plane = c.Ho * c.Wo;
  p.gs_n = c.G * c.Og * p.plane; p.xs_n = c.G * c.Cg * p.plane;
  p.ws_g = c.ws_g; p.ws_o = c.ws_o; p.ws_c = c.ws_c; p.ws_kh = c.ws_kh; p.ws_kw = c.ws_kw;
  p.w_elems = (int32_t)plan->w_elems;
  p.pitch = c.Wo + std::max(1, std::max(c.pw, c.KW - 1 - c.pw));     // at least one zero column between rows
  const int cx = (c.KH * c.KW <= 3) ? 64 : 32, halo = c.KH - 1;
  // rows per chunk: about 200 staged pixels per channel, a bounded number of staging batches per thread, and
  // both tiles within LDS
  const int vec = (c.Wo % 4 == 0) ? 4 : (c.Wo % 2 == 0) ? 2 : 1;
  // windows with a row extent go to the kernel that derives its source rows from the chunk's position and keeps
  // two chunks in LDS (one being multiplied, one being staged); the others look rows up in a table
  const int budget = kF32Items * vec * 256;        // table kernel: floats per tensor and chunk
  int trk = std::max(1, 200 / p.pitch);
  if (direct && c.Ho * p.pitch <= 256) trk = c.Ho;     // small images whole
  if (c.KH > 1) trk = std::min(trk, c.Ho);
  auto pitch_of = [&](int elems) { int v = (elems + 3) & ~3; return ((v >> 2) & 1) ? v : v + 4; };   // 4 * odd
  auto lds_need = [&](int t) {
    if (direct)      // both buffers, the spare 16 bytes
      return (int64_t)2 * (64 * pitch_of(((t * p.pitch + 3) & ~3) + 4) + cx * pitch_of((t + halo) * p.pitch + kGuardF + 8)) * 4 + 4096;
    return (int64_t)64 * (t * p.pitch + 16) * 4 + (int64_t)cx * ((t + halo) * p.pitch + halo * p.pitch + 32) * 4;
  };
  // staging items of that kernel: whole rows of 7 or 14 pixels, else `vec` pixels; 4 threads per G channel and
  // 256 / cx per X channel share a channel's items
  const int mode = (c.Wo == 7 || c.Wo == 14) ? c.Wo : vec;
  const int ni_cap = (mode == 7 ? 4 : mode == 14 ? 2 : 7) * kRowsBatches;
  auto items_g = [&](int t) { return (t * (c.Wo / mode) + 3) / 4; };
  auto items_x = [&](int t) { return ((t + halo) * (c.Wo / mode) + 256 / cx - 1) / (256 / cx); };
  auto over = [&](int t) {
    if (direct) return lds_need(t) > 160 * 1024 || std::max(items_g(t), items_x(t)) > ni_cap || t + halo > 254;
    return 64 * (t + halo) * c.Wo > budget || lds_need(t) > 140 * 1024;
  };
  while (trk > 1 && over(trk)) --trk;
  if (over(trk)) return false;
  if (c.KH > 1) {
    p.cpi = (c.Ho + trk - 1) / trk;
    trk = (c.Ho + p.cpi - 1) / p.cpi;
    p.n_chunks = c.N * p.cpi;
  } else {
    trk = std::min(trk, p.rows_total);
    p.n_chunks = (p.rows_total + trk - 1) / trk;
  }
  p.TRK = trk;
  p.n_xrows = trk + halo;
  p.CP = (p.TRK * p.pitch + 3) & ~3;
  if (direct) {
    // the last k-step reads G up to CP - 1 and X up to n_xrows * pitch + 7 (its guard included)
    p.CPg = pitch_of(p.CP + 4);
    p.CPp = pitch_of(p.n_xrows * p.pitch + kGuardF + 8);
  } else {
    p.CPp = (std::max(p.CP, p.n_xrows * p.pitch) + halo * p.pitch + c.KW + kGuardF + 4 + 3) & ~3;
    if (((p.CPp >> 2) & 1) == 0) p.CPp += 4;
    p.CPg = (p.CP + 4 + 3) & ~3;
    if (((p.CPg >> 2) & 1) == 0) p.CPg += 4;
  }
  p.items = 64 * p.n_xrows * (c.Wo / vec);
  p.magic_w2 = magic_of(c.Wo / vec);
  p.magic_rw2 = magic_of(p.n_xrows * (c.Wo / vec));
  p.n_oblk = (c.Og + 63) / 64;
  p.n_cblk = (c.Cg + cx - 1) / cx;
  const int tiles = c.G * p.n_oblk * p.n_cblk;
  p.n_tiles = tiles;
  p.ct = cx / 32;
  p.slots = 8 * p.ct * c.KH * c.KW;
  const int target = plan->opt.dw_workgroups > 0 ? plan->opt.dw_workgroups : 256;
  int splits = std::max(1, std::min(p.n_chunks, target / std::max(1, tiles)));
  while (splits > 1 && (int64_t)splits * tiles * p.slots * 1024 > (40ll << 20)) splits /= 2;
  p.chunks_per_split = (p.n_chunks + splits - 1) / splits;
  p.rows_per_split = p.chunks_per_split * p.TRK;
  p.n_splits = (p.n_chunks + p.chunks_per_split - 1) / p.chunks_per_split;
  p.lds_x_off = 64 * p.CPg * 4;
  p.lds_tab_off = p.lds_x_off + cx * p.CPp * 4;
  p.lds_bytes = p.lds_tab_off + ((2 * 2 * p.n_xrows * 4 + 15) & ~15);     // two row tables (current and next chunk)
  if (direct) {
    p.mode = mode;
    p.direct = 1;
    p.ni_g = items_g(p.TRK);
    p.ni_x = items_x(p.TRK);
    p.magic_w2 = magic_of(c.Wo / mode);
    p.magic_cpi = magic_of(p.cpi);
    p.lds_buf = p.lds_x_off + cx * p.CPp * 4;
    p.lds_tab_off = 2 * p.lds_buf;            // the 4 KB that retired items write to
    // (the final sum of the two halves needs 4 waves x 2*ct*taps accumulators x 1 KB of LDS)
    p.lds_bytes = std::max(p.lds_tab_off + 4096, 4 * 2 * p.ct * c.KH * c.KW * 1024);
    return p.lds_bytes <= 160 * 1024;
  }
  return p.lds_bytes <= 144 * 1024 && 64 * p.CPp < (1 << 30) && p.n_xrows <= 256 && p.n_xrows <= 256 &&
         (int64_t)64 * p.n_xrows * c.Wo * std::max(c.Wo, p.n_xrows * c.Wo) < (1ll << 32);
}

// Windows with a row extent take the kernel with the alternating wave halves when their rows fit its item lists,
// else (and all other windows) the kernel that looks its rows up in a table.
bool fill_dw_f32(const syno_plan* plan, DwParams& p) {
  if (plan->conv.KH == 3 && fill_dw_f32_as(plan, p, true)) return true;
  return fill_dw_f32_as(plan, p, false);
}

bool fill_any(const syno_plan* plan, DwParams& p) {
  return plan->in_dtype == SYNO_BF16 ? fill_dw(plan, p) : fill_dw_f32(plan, p);
}

}  // namespace

bool mfma_dw_supports(const syno_plan* p) {
  if (!p->conv_like) return false;
  if (p->in_dtype != SYNO_BF16 && p->in_dtype != SYNO_F32) return false;
  const ConvLike& c = p->conv;
  if (c.sh != 1 || c.sw != 1 || c.w_wrap) return false;
  // windows: 1, 3 or 5 along an axis, at most 9 taps (each tap is a set of accumulators); a 5-wide window along the
  // row only with fp32 inputs (the bf16 kernels cut their shifted fragments for 3-wide windows)
  if (c.KH != 1 && ((c.KH != 3 && c.KH != 5) || c.h_wrap || c.ph != c.KH / 2 || c.ws_kh < 0)) return false;
  if (c.Wi != c.Wo || c.Hi != c.Ho) return false;
  if (c.KW != 1 && c.KW != 3 && !(c.KW == 5 && p->in_dtype == SYNO_F32)) return false;
  if (c.KH * c.KW > 9) return false;
  if (c.pw != c.KW / 2) return false;
  if (c.ws_kw < 0 || (c.Og == 1 && c.Cg == 1)) return false;
  DwParams dp;
  return fill_any(p, dp);
}

void mfma_dw_configure(syno_plan* plan) {
  DwParams dp;
  Launch& L = plan->launch[SYNO_BWD_WEIGHT];
  static_assert(sizeof(DwParams) <= sizeof(L.params), "parameter record does not fit");
  L.params_ready = fill_any(plan, dp);
  memcpy(L.params, &dp, sizeof dp);
  L.variant = 0;
  // one 64 x 32*ct x taps tile of fp32 sums per workgroup (whole tiles also where Og or Cg end inside one)
  L.workspace = dp.n_splits == 1 ? 0 : (size_t)dp.n_splits * dp.n_tiles * dp.slots * 1024;
}

std::string mfma_dw_describe(const syno_plan* plan) {
  if (!plan->launch[SYNO_BWD_WEIGHT].params_ready) return "unconfigured";
  DwParams p;
  memcpy(&p, plan->launch[SYNO_BWD_WEIGHT].params, sizeof p);
  char b[256];
  snprintf(b, sizeof b, "rows/chunk=%d(+%d) pitch=%d chunks=%d splits=%d grid=%d lds=%dB", p.TRK, p.KH - 1, p.pitch, p.n_chunks,
           p.n_splits, p.G * p.n_oblk * p.n_cblk * p.n_splits, p.lds_bytes);
  return b;
}

namespace {
// Launch of one instantiation; the opt-in to more than 64 KB of dynamic LDS is made once per instantiation.
template <typename K, typename T>
void launch_dw_kernel(K kernel, int grid, const DwParams& p, const T* G, const T* X, float* dst, hipStream_t stream,
                      int threads = 256) {
  static const hipError_t lds_opt_in =
      hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (lds_opt_in != hipSuccess) return;
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), p.lds_bytes, stream, p, G, X, dst);
}
}  // namespace

// A = G (upstream gradient), B = X, out = dW (fp32), ws = n_splits partial copies of dW.
syno_status launch_mfma_dw(const syno_plan* plan, const void* A, const void* B, void* out, void* ws, hipStream_t stream) {
  if (!plan->launch[SYNO_BWD_WEIGHT].params_ready) return SYNO_ERR_UNSUPPORTED;
  DwParams p;
  memcpy(&p, plan->launch[SYNO_BWD_WEIGHT].params, sizeof p);
  if (!ws && p.n_splits > 1) return SYNO_ERR_WORKSPACE;
  const int grid = p.G * p.n_oblk * p.n_cblk * p.n_splits;
  float* const dst = p.n_splits == 1 ? static_cast<float*>(out) : static_cast<float*>(ws);
  using std::integral_constant;
  auto by_window = [&](auto go) {
    if (p.KH == 3 && p.KW == 3) go(integral_constant<int, 3>{}, integral_constant<int, 3>{}, integral_constant<int, 1>{});
    else if (p.KH == 5) go(integral_constant<int, 5>{}, integral_constant<int, 1>{}, integral_constant<int, 1>{});
    else if (p.KW == 5) go(integral_constant<int, 1>{}, integral_constant<int, 5>{}, integral_constant<int, 1>{});
    else if (p.KH == 3) go(integral_constant<int, 3>{}, integral_constant<int, 1>{}, integral_constant<int, 2>{});
    else if (p.KW == 3) go(integral_constant<int, 1>{}, integral_constant<int, 3>{}, integral_constant<int, 2>{});
    else go(integral_constant<int, 1>{}, integral_constant<int, 1>{}, integral_constant<int, 2>{});
  };
  if (plan->in_dtype == SYNO_F32) {
    const float* Gf = static_cast<const float*>(A);
    const float* Xf = static_cast<const float*>(B);
    by_window([&](auto kh_c, auto kw_c, auto ct_c) {
      constexpr int kh = decltype(kh_c)::value, kw = decltype(kw_c)::value, ct = decltype(ct_c)::value;
      if (kh == 3 && p.direct) {
        if constexpr (kh == 3) {
        if (p.mode == 4) launch_dw_kernel(dw_rows_f32<kw, ct, 4>, grid, p, Gf, Xf, dst, stream, kRowsThreads);
        else if (p.mode == 7) launch_dw_kernel(dw_rows_f32<kw, ct, 7>, grid, p, Gf, Xf, dst, stream, kRowsThreads);
        else if (p.mode == 14) launch_dw_kernel(dw_rows_f32<kw, ct, 14>, grid, p, Gf, Xf, dst, stream, kRowsThreads);
        else if (p.mode == 2) launch_dw_kernel(dw_rows_f32<kw, ct, 2>, grid, p, Gf, Xf, dst, stream, kRowsThreads);
        else launch_dw_kernel(dw_rows_f32<kw, ct, 1>, grid, p, Gf, Xf, dst, stream, kRowsThreads);
        }
      } else {
        if (p.W % 4 == 0) launch_dw_kernel(dw_mfma_f32<kh, kw, ct, 4>, grid, p, Gf, Xf, dst, stream);
        else if (p.W % 2 == 0) launch_dw_kernel(dw_mfma_f32<kh, kw, ct, 2>, grid, p, Gf, Xf, dst, stream);
        else launch_dw_kernel(dw_mfma_f32<kh, kw, ct, 1>, grid, p, Gf, Xf, dst, stream);
      }
    });
  } else {
    const uint16_t* G = static_cast<const uint16_t*>(A);
    const uint16_t* X = static_cast<const uint16_t*>(B);
    by_window([&](auto kh_c, auto kw_c, auto ct_c) {
      constexpr int kh = decltype(kh_c)::value, kw = decltype(kw_c)::value, ct = decltype(ct_c)::value;
      if constexpr (kw == 5) {
        return;                 // (not instantiated: mfma_dw_supports refuses it)
      } else {
      bool taken = false;
      if constexpr (kh == 3) {
        taken = p.direct != 0;
        if (p.direct && p.mode == 7) launch_dw_kernel(dw_rows_bf16<kw, ct, 7>, grid, p, G, X, dst, stream, kRowsThreads);
        else if (p.direct) launch_dw_kernel(dw_rows_bf16<kw, ct, 14>, grid, p, G, X, dst, stream, kRowsThreads);
      }
      if (taken) return;
      if (p.W % 4 == 0) launch_dw_kernel(dw_mfma_bf16<kh, kw, ct, 4>, grid, p, G, X, dst, stream);
      else if (p.W % 2 == 0) launch_dw_kernel(dw_mfma_bf16<kh, kw, ct, 2>, grid, p, G, X, dst, stream);
      else launch_dw_kernel(dw_mfma_bf16<kh, kw, ct, 1>, grid, p, G, X, dst, stream);
      }
    });
  }
  // many splits of a small dW: one block per slot keeps the device busy; few splits, or a dW with at least one 16x16
  // tile per compute unit: one block per tile with all its taps writes dW in whole lines
  if (p.n_splits == 1) {
    // (written by the contraction itself)
  } else if (p.n_splits > 4 && p.n_tiles * (p.slots / (p.KH * p.KW)) < 256)
    hipLaunchKernelGGL(dw_reduce_slots, dim3(p.n_tiles * p.slots), dim3(256), 0, stream, p,
                       reinterpret_cast<const float4*>(ws), static_cast<float*>(out));
  else
    hipLaunchKernelGGL(dw_reduce_tiles, dim3(p.n_tiles * (p.slots / (p.KH * p.KW))), dim3(256), 0, stream, p,
                       reinterpret_cast<const float4*>(ws), static_cast<float*>(out));
  return hipGetLastError() == hipSuccess ? SYNO_OK : SYNO_ERR_HIP;
}

}  // namespace syno
