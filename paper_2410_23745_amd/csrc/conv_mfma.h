// MFMA contraction family, device side: parameter record, the kernel template, its tile variants and
// the launch helper.  Included by the host logic and by the translation units that instantiate the
// variants (several files, so that they compile in parallel).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

namespace syno {
struct MfmaParams {
  // problem, in forward terms
  int32_t G, Og, Cg, Ho, Wo, Hi, Wi, KH, KW, ph, pw;
  int32_t sh, sw;                     // Stride below the window: output (h, w), tap (kh, kw) reads input (sh*h+kh-ph, sw*w+kw-pw)
  int32_t rows_total;                 // N*Ho output rows
  int32_t h_wrap, h_shift, h_shift_g; // cyclic rows: input row = (h + h_shift + h_shift_g*g) mod Hi  (KH = 1)
  int32_t xs_n, xs_c;                 // source strides: image, channel (rows are Wi apart, columns adjacent)
  int32_t os_n, os_o;                 // result strides: image, channel
  int32_t ws_g, ws_o, ws_c, ws_kh, ws_kw, w_base;
  uint32_t probe_lo, probe_hi;        // optional clock probe (device address of 4 x int64 per workgroup; 0: none)
  // tiling
  int32_t TR, BN, KC, n_mblocks, n_nblocks, n_chunks;
  int32_t n_slots, Wp, cgrps;
  int32_t vx;                         // pixels per X item: 4, or 1 for rows narrower than 4 (slow path: each element load is waited for)
  int32_t vpr;                        // X items that cover one input row (the last one may overlap its neighbour)
  int32_t w_row;                      // LDS weight row pitch (elements)
  int32_t lds_w_off, lds_tab_off, lds_bytes;
  int32_t w_block;                    // bf16: elements of one packed weight block (KH*KW*BN*w_row)
  // ceil(2^32/d) for the divisors the kernel needs (exact quotients for n*d < 2^32, which the host checks)
  uint32_t m_wo, m_ho, m_vpr, m_pcg, m_per_o, m_khw, m_kw;
  int32_t wf;                         // bf16 single-chunk variant: taps per channel when the weights are read unpacked, else 0
  int32_t wt;                         // fp32 backward-data: the weights are first transposed into the workspace
  int32_t wadj;                       // fp32 backward-data, 3x3 window, weights in the forward layout [o][c][9 taps]: the
                                      // adjoint's block is transposed and its taps reversed on the way into LDS (no copy)
  int32_t ts_g, ts_o, ts_c, ts_kh, ts_kw;   // ... from a tensor with these strides
  int32_t U;                          // window taps along w per row-step (selects the instantiation)
  int32_t ksplit, chunks_per_split;   // workgroups per output tile, each summing a range of chunks (1: no split)
  int32_t split_stride;               // ksplit > 1: elements between the partial results (fp32, laid out like the result)
  // Workgroups are handed round-robin to the 8 XCDs, each with an L2 of its own.  When xcd_m > 0 the tiles of one
  // (group, split) plane are dealt so that XCD x = xm*xcd_n + xn works on an (n_mblocks/xcd_m) x (n_nblocks/xcd_n)
  // rectangle of tiles: it reads 1/xcd_m of the source rows and 1/xcd_n of the weights (xcd_m * xcd_n = 8).  0: the
  // plain order (weight panels fastest).  Inside its rectangle an XCD takes the panels of one row of tiles first, or
  // (xcd_rows_first) the rows of tiles of one panel first.
  int32_t xcd_m, xcd_n, xcd_rows_first;
};

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
// four adjacent pixels of one channel as they lie in memory (rows start at any element, so only element alignment)
typedef float f32x4_unaligned __attribute__((ext_vector_type(4), aligned(4)));
typedef uint16_t bf16x4_unaligned __attribute__((ext_vector_type(4), aligned(2)));

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
    const int seg_slots = (seg_rows - 1) * p.sh + p.KH;      // consecutive input rows, first one sh*h - ph
    if (s < s0 + seg_slots) {
      const int r = h * p.sh + (s - s0) - p.ph;
      return (r >= 0 && r < p.Hi) ? n * p.xs_n + r * p.Wi : -1;
    }
    s0 += seg_slots;
    rho += seg_rows;
  }
  return -1;
}

// First slot of output row i of the block (tap kh adds kh slots): a run of r rows of one image takes (r-1)*sh + KH
// slots, so every image boundary before the row adds KH - sh to sh*i.
__device__ __forceinline__ int slot_of_row(const MfmaParams& p, int R0, int i) {
  if (p.h_wrap) return i;
  return i * p.sh + (p.KH - p.sh) * (fdiv(R0 + i, p.m_ho) - fdiv(R0, p.m_ho));
}

// f(integral_constant<int, I>) for I = 0 .. N-1
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// BF = false: fp32 inputs, CI = 4, v_mfma_f32_16x16x4_f32  (A: lane -> row l%16, k = l/16).
// BF = true : bf16 inputs, CI = 8, v_mfma_f32_16x16x32_bf16 (A: lane -> row l%16, k = 8*(l/16)..+7);
//             `Wv` is the packed copy.
// WNAT (fp32 only): the weight block of one output channel, [KC][KH][KW], is contiguous and 16-byte
//             aligned in memory, so it is staged with 16-byte loads instead of element by element.
// KCB: bf16 only: channels per chunk (a compile-time constant there, since it fixes the tap offsets in LDS)
// WF:  bf16: > 0 = the weights are read as they lie in memory ([o][c][WF taps], the forward layout) and re-ordered
//      on their way into LDS, instead of coming from the packed copy; < 0 = the same for backward-data: the
//      single-chunk variant brings its whole block in at the start, the others (9 taps only) chunk by chunk
// U:   window taps along w handled per "row-step" (3 when KW = 3, else 1): the operands of the U taps sit at
//      compile-time LDS offsets from one per-lane address, so addresses advance once per row-step.
// WK:  waves that share one output tile and split each chunk's k-steps among themselves (for shapes whose
//      per-SIMD share of the output is only a few MFMA tiles: a wave then still issues TM*TN MFMAs per
//      LDS round trip); their accumulators are added through LDS at the end.
template <bool BF, bool WNAT, int WM, int WN, int WK, int TM, int TN, int XI, int WI, bool ONE, int KCB, int U, int WF, bool OUTBF>
__global__ __launch_bounds__(WM* WN* WK * 64) void conv_mfma(const MfmaParams p, const void* __restrict__ Xv,
                                                         const void* __restrict__ Wv, void* __restrict__ out) {
  constexpr int NT = WM * WN * WK * 64;
  constexpr int BN = WN * TN * 16;
  constexpr int CI = BF ? 8 : 4;
  constexpr int CG_STEP = BF ? 4 : 1;        // channel groups one MFMA consumes
  using XT = std::conditional_t<BF, uint16_t, float>;
  using XV = std::conditional_t<BF, bf16x4_unaligned, f32x4_unaligned>;   // 4 pixels of one channel
  using Frag = std::conditional_t<BF, bf16x8, float>;
  constexpr bool W16 = BF || WNAT;           // weights move in 16-byte pieces
  using WReg = std::conditional_t<W16, uint4, float>;
  extern __shared__ __align__(16) unsigned char smem[];
  float4* xl = reinterpret_cast<float4*>(smem);
  int* slot_src = reinterpret_cast<int*>(smem + p.lds_tab_off);

  long long* const probe = reinterpret_cast<long long*>(((unsigned long long)p.probe_hi << 32) | p.probe_lo);
  if (probe && threadIdx.x == 0) {
    probe[(long long)blockIdx.x * 4 + 0] = wall_clock64();
    probe[(long long)blockIdx.x * 4 + 1] = clock64();
  }
  const int tid = threadIdx.x, lane = tid & 63;
  const int widx = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in an SGPR
  const int wk = widx / (WM * WN), wtile = widx - wk * (WM * WN);
  const int wn = wtile / WM;
  // wave widx runs on SIMD widx % 4: rotate the wave rows so that the fuller ones spread over the SIMDs,
  // also among the waves that split K
  const int wm = (wtile + wn + ((wk * WM * WN) >> 2)) % WM;
  int bid = blockIdx.x, nb, mb;
  if (p.xcd_m > 0) {
    // (a plane holds a multiple of 8 tiles, so the low three bits of its local index name the XCD)
    const int tiles = p.n_mblocks * p.n_nblocks;
    const int plane = bid / tiles, local = bid - plane * tiles;
    const int xcd = local & 7, idx = local >> 3;
    const int sm = p.n_mblocks / p.xcd_m, sn = p.n_nblocks / p.xcd_n;
    const int xm = xcd / p.xcd_n, xn = xcd - xm * p.xcd_n;
    const int im = p.xcd_rows_first ? idx % sm : idx / sn;
    mb = xm * sm + im; nb = xn * sn + (p.xcd_rows_first ? idx / sm : idx - im * sn);
    bid = plane * p.n_mblocks;
  } else {
    nb = bid % p.n_nblocks; bid /= p.n_nblocks;
    mb = bid % p.n_mblocks;
  }
  int g = bid / p.n_mblocks, ksp = 0;
  if (p.ksplit > 1) { ksp = g / p.G; g -= ksp * p.G; }
  const int R0 = mb * p.TR;
  const int rows = min(p.TR, p.rows_total - R0);
  const int KHW = p.KH * p.KW;

  for (int s = tid; s < p.n_slots; s += NT) slot_src[s] = slot_source(p, R0, rows, g, s);
  __syncthreads();

  // ---- loop-invariant descriptors of what this thread stages per chunk
  const XT* Xg = reinterpret_cast<const XT*>(Xv) + (int64_t)g * p.Cg * p.xs_c;
  // An X item is vx = 4 adjacent pixels of one input row x CI channels: CI vector loads, then one 16-byte
  // LDS write per pixel.  A row's last item is moved left to end at the row's end when Wi is no multiple
  // of 4.  (vx = 1: one pixel per item, element loads.)
  int x_goff[XI], x_loff[XI], x_cg[XI];
  {
    const int per_cg = p.n_slots * p.vpr, total = p.cgrps * per_cg;
#pragma unroll
    for (int k = 0; k < XI; ++k) {
      const int idx = tid + k * NT;
      const int cg = fdiv(idx, p.m_pcg), rem = idx - cg * per_cg;
      const int s = fdiv(rem, p.m_vpr), x = min((rem - s * p.vpr) * p.vx, p.Wi - p.vx);
      const int src = idx < total ? slot_src[s] : -1;
      x_goff[k] = src >= 0 ? src + x + cg * CI * p.xs_c : -1;
      x_loff[k] = (cg * p.n_slots + s) * p.Wp + x + p.pw;
      x_cg[k] = cg * CI;
    }
  }
  int w_goff[WI], w_meta[WI];   // fp32 meta: LDS dword offset | local channel << 20 | zero-fill << 29 | unused << 30
  const float* Wg32 = nullptr;
  const uint4* Wg16 = nullptr;
  // fp32: one weight element per item, gathered with the operator's strides into [o][c*KHW+tap].
  // bf16: 16-byte pieces of this block's packed image, copied as they are.
  // bf16, WF > 0: weights as they lie in memory.  An item is 8 channels x WF taps of one output channel of the
  // chunk (WF adjacent 16-byte loads); on the way into LDS it is re-ordered into one 16-byte piece per tap.
  constexpr int kAdjPairs = (WI * 4) / 9;      // (fp32, adjoint from the forward layout) pairs of 9 taps a thread's weight registers hold
  constexpr int OCT = BF ? KCB / 8 : 1;                                     // channel octets per chunk
  // bf16 backward-data of a multi-chunk variant straight from forward-layout weights W[o][c][9 taps]: an item is one
  // row of the block (a forward input channel c) x one octet of the chunk's reduction channels (forward output
  // channels o): eight runs of 9 adjacent taps, a forward output-channel stride apart, each read as 16 + 2 bytes;
  // on the way into LDS they become one 16-byte piece per tap (the 8 channels of the octet), taps reversed
  constexpr bool WADJ = BF && WF < 0 && !ONE;
  static_assert(!WADJ || WF == -9, "the chunked adjoint reads runs of 9 taps");
  constexpr int WP = (BF && (WF > 0 || WADJ)) ? (BN * OCT + NT - 1) / NT : 1;   // such items per thread
  constexpr int WFA = WF > 0 ? WF : 1;
  constexpr int WIN = WADJ ? 8 * 5 : 4 * WFA;                               // dwords of one item in registers
  int wp_src[WP], wp_dst[WP], wp_c[WP];   // element offset in W at chunk 0; LDS piece index at tap 0 (-1: unused);
                                          // first channel inside the chunk | row beyond Og << 30
  const uint16_t* Wnat = nullptr;
  if constexpr (BF && WF > 0) {
    Wnat = reinterpret_cast<const uint16_t*>(Wv) + (int64_t)g * p.ws_g + (int64_t)nb * BN * p.ws_o;
#pragma unroll
    for (int k = 0; k < WP; ++k) {
      const int idx = tid + k * NT;
      const int octet = idx % OCT, ol = idx / OCT;
      wp_src[k] = ol * p.ws_o + octet * 8 * WF;
      wp_dst[k] = idx < BN * OCT ? ol * ((KCB + 8) / 8) + octet : -1;
      wp_c[k] = octet * 8 | (nb * BN + ol < p.Og ? 0 : (1 << 30));
    }
  } else if constexpr (WADJ) {
    // (p.ws_o is the forward channel stride = 9, p.ws_c the forward output-channel stride)
    Wnat = reinterpret_cast<const uint16_t*>(Wv) + (int64_t)g * p.ws_g + (int64_t)nb * BN * 9;
#pragma unroll
    for (int k = 0; k < WP; ++k) {
      // adjacent lanes take adjacent rows: their runs of one forward output channel are adjacent in memory (18 bytes
      // each), and their 16-byte pieces go to LDS rows one pitch apart, the fragment reads' conflict-free pattern
      const int idx = tid + k * NT;
      const int ol = idx % BN, octet = idx / BN;
      wp_src[k] = ol * 9 + octet * 8 * p.ws_c;
      wp_dst[k] = idx < BN * OCT ? ol * ((KCB + 8) / 8) + octet : -1;
      wp_c[k] = octet * 8 | (nb * BN + ol < p.Og ? 0 : (1 << 30));
    }
  } else if constexpr (BF && WF != 0) {
    // (backward-data of the single-chunk variant: the block is brought in once, below)
  } else if constexpr (BF) {
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
    if (p.wadj) {
      // adjoint straight from W[o][c][9 taps] (this kernel's channel = o, its output channel = c): an item is the 9
      // taps of one (output channel, channel) pair, 36 adjacent bytes.  A wave takes 16 adjacent output channels x 4
      // adjacent channels at a time: 576 contiguous bytes per channel on the memory side, and on the LDS side the
      // pattern of a B-fragment read (16 rows x 4 steps of 9 dwords), which the row pitch keeps free of bank conflicts
#pragma unroll
      for (int k = 0; k < WI; ++k) {
        const int idx = tid + k * NT;
        const int rest = idx >> 6;
        const int r = (idx & 15) + 16 * (rest % (BN / 16)), cl = ((idx >> 4) & 3) + 4 * (rest / (BN / 16));
        const bool in = k < kAdjPairs && idx < BN * p.KC;
        w_goff[k] = (in && nb * BN + r < p.Og) ? cl * p.ws_c + r * 9 : -1;   // element offset at chunk 0
        w_meta[k] = in ? r * p.w_row + cl * 9 : -1;                          // LDS float index of the pair's first tap
      }
    } else {
#pragma unroll
    for (int k = 0; k < WI; ++k) {
      const int idx = tid + k * NT;
      const int o = fdiv(idx, p.m_per_o), e4 = idx - o * per_o4;
      const bool ok = idx < total && nb * BN + o < p.Og;
      w_goff[k] = ok ? o * p.ws_o + e4 * 4 : -1;                 // element offset
      w_meta[k] = idx < total ? (o * p.w_row + e4 * 4) >> 2 : -1; // LDS float4 index
    }
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
  int a_base[TM];                                   // LDS byte address of the lane's A operand at tap (0,0), channel group 0
#pragma unroll
  for (int t = 0; t < TM; ++t) {
    int m = (my_first + t) * 16 + (lane & 15);
    if (t >= my_tiles || m >= block_px) m = 0;
    const int i = fdiv(m, p.m_wo), w = m - i * p.Wo;
    const int px = slot_of_row(p, R0, i) * p.Wp + w * p.sw;
    a_base[t] = BF ? (px + (lane >> 4) * cg_stride) * 16 : px * 16 + (lane >> 4) * 4;
  }
  int b_base[TN];                                   // same for the B operand (weights)
#pragma unroll
  for (int u = 0; u < TN; ++u) {
    const int ol = (wn * TN + u) * 16 + (lane & 15);
    b_base[u] = p.lds_w_off + (BF ? (ol * p.w_row + (lane >> 4) * 8) * 2 : (ol * p.w_row + (lane >> 4) * KHW) * 4);
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

  XV xr[XI][CI];
  WReg wr[WI];
  uint32_t win[WP][WIN];         // (bf16 weights read as they lie in memory only)
  // dword I of the weight registers taken as one flat array (16-byte pieces only)
  auto wcomp = [&](auto i_c) -> uint32_t& {
    constexpr int I = decltype(i_c)::value;
    if constexpr (!W16) return win[0][0];
    else if constexpr (I % 4 == 0) return wr[I / 4].x;
    else if constexpr (I % 4 == 1) return wr[I / 4].y;
    else if constexpr (I % 4 == 2) return wr[I / 4].z;
    else return wr[I / 4].w;
  };
  // Loads use a wave-uniform base plus 32-bit byte offsets.  Items without a source read offset 0 (any
  // valid address) and are simply not written to LDS, so the common path has no per-load predicate.
  const bool chan_tail = (p.Cg % p.KC) != 0;
  const char* xbase = reinterpret_cast<const char*>(Xg);
  // A chunk's requests are dealt into kSlices slices (slice_c < 0: all of them).  The first chunk goes out
  // at once; the following ones slice by slice between the first k-steps of the chunk before, because a
  // burst of everything holds the wave at the memory pipeline's queues instead of at its MFMAs.
  constexpr int kSlices = WK == 1 ? 2 : 1;     // (K-split waves run too few k-steps per chunk to spread anything)
  auto load1 = [](const void* src) { return *reinterpret_cast<const XT*>(src); };   // (no arithmetic on the value here: that would wait for it)
  auto fetch = [&](int ch, auto slice_c) {
    constexpr int slice = decltype(slice_c)::value;
    auto want = [&](int k) { return slice < 0 || slice == k % kSlices; };
    const int c0 = ch * p.KC;
    if (!chan_tail) {
#pragma unroll
      for (int k = 0; k < XI; ++k) {
        const uint32_t o = (uint32_t)(max(x_goff[k], 0) + c0 * p.xs_c) * (uint32_t)sizeof(XT);
#pragma unroll
        for (int j = 0; j < CI; ++j)
          if (want(k * CI + j)) {
            const char* src = xbase + (o + (uint32_t)(j * p.xs_c) * (uint32_t)sizeof(XT));
            if (p.vx == 1) {
              xr[k][j] = XV{load1(src), 0, 0, 0};   // (whole register written: nothing to merge after the load)
              continue;
            }
            xr[k][j] = *reinterpret_cast<const XV*>(src);
          }
      }
    } else {
#pragma unroll
      for (int k = 0; k < XI; ++k)
#pragma unroll
        for (int j = 0; j < CI; ++j) {
          if (!want(k * CI + j)) continue;
          const int c = c0 + x_cg[k] + j;
          xr[k][j] = XV(0);
          if (x_goff[k] >= 0 && c < p.Cg) {
            const XT* src = Xg + x_goff[k] + (int64_t)(c0 + j) * p.xs_c;
            if (p.vx == 1) xr[k][j] = XV{load1(src), 0, 0, 0};   // (whole register written: nothing to merge after the load)
            else xr[k][j] = *reinterpret_cast<const XV*>(src);
          }
        }
    }
    if constexpr (BF && WF > 0) {
      // unconditional loads (what has no source reads the block's first elements and is zeroed when staged)
      typedef uint32_t u32x4_unaligned __attribute__((ext_vector_type(4), aligned(2)));
#pragma unroll
      for (int k = 0; k < WP; ++k) {
        const bool live = wp_dst[k] >= 0 && !(wp_c[k] >> 30) && c0 + (wp_c[k] & 0xffff) < p.Cg;
        const uint16_t* src = Wnat + (live ? wp_src[k] + c0 * WF : 0);
#pragma unroll
        for (int q = 0; q < WFA; ++q)
          if (want(XI * CI + k * WFA + q)) {
            const u32x4_unaligned v = *reinterpret_cast<const u32x4_unaligned*>(src + q * 8);
            win[k][4 * q + 0] = v[0]; win[k][4 * q + 1] = v[1]; win[k][4 * q + 2] = v[2]; win[k][4 * q + 3] = v[3];
          }
      }
    } else if constexpr (WADJ) {
      typedef uint32_t u32x4_unaligned __attribute__((ext_vector_type(4), aligned(2)));
#pragma unroll
      for (int k = 0; k < WP; ++k) {
        // (the reduction length is a multiple of 8, so an octet that starts inside it lies inside it)
        const bool live = wp_dst[k] >= 0 && !(wp_c[k] >> 30) && c0 + (wp_c[k] & 0xffff) < p.Cg;
        const uint16_t* src = Wnat + (live ? (int64_t)wp_src[k] + (int64_t)c0 * p.ws_c : 0);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint16_t* run = src + (int64_t)e * p.ws_c;
          if (want(XI * CI + k * 16 + 2 * e)) {
            const u32x4_unaligned v = *reinterpret_cast<const u32x4_unaligned*>(run);
            win[k][5 * e + 0] = v[0]; win[k][5 * e + 1] = v[1]; win[k][5 * e + 2] = v[2]; win[k][5 * e + 3] = v[3];
          }
          if (want(XI * CI + k * 16 + 2 * e + 1)) win[k][5 * e + 4] = run[8];
        }
      }
    } else if constexpr (BF && WF != 0) {
    } else if constexpr (BF) {
      const uint4* src = Wg16 + (int64_t)ch * (p.w_block >> 3);
#pragma unroll
      for (int k = 0; k < WI; ++k)
        if (want(XI * CI + k)) wr[k] = w_goff[k] >= 0 ? src[w_goff[k]] : make_uint4(0, 0, 0, 0);
    } else if constexpr (WNAT) {
      // (the planner only picks this path when Cg is a multiple of KC, so no channel tail here)
      if (p.wadj) {
        if constexpr (kAdjPairs > 0)
          static_for<0, kAdjPairs>([&](auto k_c) {
            constexpr int k = decltype(k_c)::value;
            if (!want(XI * CI + k)) return;
            // (pairs without a source read the block's first taps and are written as zeros)
            const float* src = Wg32 + max(w_goff[k], 0) + (int64_t)c0 * p.ws_c;
            const f32x4_unaligned a = *reinterpret_cast<const f32x4_unaligned*>(src);
            const f32x4_unaligned b = *reinterpret_cast<const f32x4_unaligned*>(src + 4);
            const float last = src[8];
            static_for<0, 4>([&](auto i_c) { wcomp(std::integral_constant<int, 9 * k + decltype(i_c)::value>{}) = __float_as_uint(a[decltype(i_c)::value]); });
            static_for<0, 4>([&](auto i_c) { wcomp(std::integral_constant<int, 9 * k + 4 + decltype(i_c)::value>{}) = __float_as_uint(b[decltype(i_c)::value]); });
            wcomp(std::integral_constant<int, 9 * k + 8>{}) = __float_as_uint(last);
          });
      } else {
#pragma unroll
      for (int k = 0; k < WI; ++k)
        if (want(XI * CI + k))
          wr[k] = w_goff[k] >= 0 ? *reinterpret_cast<const uint4*>(Wg32 + w_goff[k] + (int64_t)c0 * p.ws_c)
                                 : make_uint4(0, 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int k = 0; k < WI; ++k) {
        if (!want(XI * CI + k)) continue;
        const int cl = (w_meta[k] >> 20) & 511;
        wr[k] = (!(w_meta[k] >> 29) && c0 + cl < p.Cg) ? Wg32[w_goff[k] + (int64_t)c0 * p.ws_c] : 0.f;
      }
    }
  };
  auto stage = [&](int ch) {
    (void)ch;
#pragma unroll
    for (int k = 0; k < XI; ++k)
      if (x_goff[k] >= 0) {
        uint4* dst = reinterpret_cast<uint4*>(xl) + x_loff[k];
        if constexpr (BF) {
          // pixel i of channel j is half (i&1) of dword (i>>1) of xr[k][j]; a pixel's 8 channels go out together
          uint2 d[CI];
#pragma unroll
          for (int j = 0; j < CI; ++j) d[j] = __builtin_bit_cast(uint2, xr[k][j]);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            if (i >= p.vx) break;
            const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;   // high or low halves of (second, first)
            auto w = [&](int j) { return (i >> 1) ? d[j].y : d[j].x; };   // the dword of channel j that holds pixel i
            uint4 v;
            v.x = __builtin_amdgcn_perm(w(1), w(0), sel);
            v.y = __builtin_amdgcn_perm(w(3), w(2), sel);
            v.z = __builtin_amdgcn_perm(w(5), w(4), sel);
            v.w = __builtin_amdgcn_perm(w(7), w(6), sel);
            dst[i] = v;
          }
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (i < p.vx) xl[x_loff[k] + i] = make_float4(xr[k][0][i], xr[k][1][i], xr[k][2][i], xr[k][3][i]);
          (void)dst;
        }
      }
    if constexpr (BF && WF > 0) {
      uint4* wl = reinterpret_cast<uint4*>(smem + p.lds_w_off);
      const int c0 = ch * p.KC;
#pragma unroll
      for (int k = 0; k < WP; ++k)
        if (wp_dst[k] >= 0) {
          const bool live = !(wp_c[k] >> 30) && c0 + (wp_c[k] & 0xffff) < p.Cg;
#pragma unroll
          for (int tap = 0; tap < WFA; ++tap) {
            uint32_t d[4];
#pragma unroll
            for (int h = 0; h < 4; ++h) {
              // channels 2h and 2h+1 of this tap: elements (2h)*WF+tap and (2h+1)*WF+tap of the 8*WF loaded ones
              const int e0 = (2 * h) * WFA + tap, e1 = (2 * h + 1) * WFA + tap;
              const uint32_t sel = ((e0 & 1) ? 0x0302u : 0x0100u) | ((e1 & 1) ? 0x07060000u : 0x05040000u);
              d[h] = live ? __builtin_amdgcn_perm(win[k][e1 >> 1], win[k][e0 >> 1], sel) : 0u;
            }
            wl[tap * BN * ((KCB + 8) / 8) + wp_dst[k]] = make_uint4(d[0], d[1], d[2], d[3]);
          }
        }
    } else if constexpr (WADJ) {
      uint4* wl = reinterpret_cast<uint4*>(smem + p.lds_w_off);
      const int c0 = ch * p.KC;
#pragma unroll
      for (int k = 0; k < WP; ++k)
        if (wp_dst[k] >= 0) {
          const bool live = !(wp_c[k] >> 30) && c0 + (wp_c[k] & 0xffff) < p.Cg;
#pragma unroll
          for (int tap = 0; tap < 9; ++tap) {
            // tap `tap` of run e is half (tap & 1) of dword tap/2 of the run (the ninth sits alone in the fifth dword)
            constexpr uint32_t lo = 0x05040100u, hi = 0x07060302u;
            const int dw = tap < 8 ? tap >> 1 : 4;
            const uint32_t sel = (tap < 8 && (tap & 1)) ? hi : lo;
            uint32_t d[4];
#pragma unroll
            for (int h = 0; h < 4; ++h)
              d[h] = live ? __builtin_amdgcn_perm(win[k][5 * (2 * h + 1) + dw], win[k][5 * (2 * h) + dw], sel) : 0u;
            wl[(8 - tap) * BN * ((KCB + 8) / 8) + wp_dst[k]] = make_uint4(d[0], d[1], d[2], d[3]);    // taps reversed
          }
        }
    } else if constexpr (BF && WF != 0) {
    } else if constexpr (BF) {
      uint4* wl = reinterpret_cast<uint4*>(smem + p.lds_w_off);
#pragma unroll
      for (int k = 0; k < WI; ++k)
        if (w_goff[k] >= 0) wl[w_goff[k]] = wr[k];
    } else if constexpr (WNAT) {
      if (p.wadj) {
        if constexpr (kAdjPairs > 0)
          static_for<0, kAdjPairs>([&](auto k_c) {
            constexpr int k = decltype(k_c)::value;
            if (w_meta[k] < 0) return;
            float* dst = reinterpret_cast<float*>(smem + p.lds_w_off) + w_meta[k];
            const bool live = w_goff[k] >= 0;
            static_for<0, 9>([&](auto i_c) {       // taps reversed
              constexpr int i = decltype(i_c)::value;
              dst[8 - i] = live ? __uint_as_float(wcomp(std::integral_constant<int, 9 * k + i>{})) : 0.f;
            });
          });
      } else {
      uint4* wl = reinterpret_cast<uint4*>(smem + p.lds_w_off);
#pragma unroll
      for (int k = 0; k < WI; ++k)
        if (w_meta[k] >= 0) wl[w_meta[k]] = wr[k];
      }
    } else {
      float* wl = reinterpret_cast<float*>(smem + p.lds_w_off);
#pragma unroll
      for (int k = 0; k < WI; ++k)
        if (!(w_meta[k] >> 30)) wl[w_meta[k] & 0xfffff] = wr[k];
    }
  };

  // ONE: the whole reduction fits one chunk, so the staging registers are dead once it is in LDS
  // (workgroups that split the reduction take chunks_per_split chunks each; the host rules out empty ranges)
  const int ch_begin = ONE ? 0 : ksp * p.chunks_per_split;
  const int n_chunks = ONE ? 1 : min(p.n_chunks, ch_begin + p.chunks_per_split);
  fetch(ch_begin, std::integral_constant<int, -1>{});
  // while the first requests travel: zero the X region once (slot edges and rows outside the image are the
  // window's zero padding and are never written afterwards); the loop's first barrier orders it before staging
  {
    const int n16 = p.cgrps * p.n_slots * p.Wp;
    for (int i = tid; i < n16; i += NT) xl[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  if constexpr (BF && WF < 0 && ONE) {
    // The same for the backward-data adjoint: the B operand's rows are the forward input channels and its
    // reduction runs over the forward output channels, taps reversed.  A thread again loads 8 channels x
    // T taps of one forward output channel o, but each element goes to its own row: [T-1-tap][c][o].
    static_assert(ONE, "only the single-chunk variant stages weights this way");
    typedef uint32_t u32x4_unaligned __attribute__((ext_vector_type(4), aligned(2)));
    constexpr int T = -WF, OCT = BN / 8, ROW = KCB + 8;
    // (p.ws_o is the forward channel stride = T, p.ws_c the forward output-channel stride)
    const uint16_t* Wt = reinterpret_cast<const uint16_t*>(Wv) + (int64_t)g * p.ws_g + (int64_t)nb * BN * T;
    uint16_t* wl = reinterpret_cast<uint16_t*>(smem + p.lds_w_off);
    for (int i = tid; i < KCB * OCT; i += NT) {
      const int octet = i % OCT, o = i / OCT;
      const bool live = o < p.Cg && nb * BN + octet * 8 < p.Og;
      uint32_t in[4 * T];
#pragma unroll
      for (int q = 0; q < T; ++q) {
        u32x4_unaligned v = {0, 0, 0, 0};
        if (live) v = *reinterpret_cast<const u32x4_unaligned*>(Wt + (int64_t)o * p.ws_c + octet * 8 * T + q * 8);
        in[4 * q + 0] = v[0]; in[4 * q + 1] = v[1]; in[4 * q + 2] = v[2]; in[4 * q + 3] = v[3];
      }
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int tap = 0; tap < T; ++tap) {
          const int e = j * T + tap;
          wl[((T - 1 - tap) * BN + octet * 8 + j) * ROW + o] = (uint16_t)((e & 1) ? in[e >> 1] >> 16 : in[e >> 1]);
        }
    }
  }
  for (int ch = ch_begin; ch < n_chunks; ++ch) {
    __syncthreads();   // everyone has finished reading the previous chunk
    stage(ch);
    __syncthreads();
    const bool more = ch + 1 < n_chunks;   // the next chunk travels while this one is computed
    bool requested = false;
    // One MFMA k-step = CI*CG_STEP channels at one tap.  A row-step is one (channel step, kh, group of U
    // taps along w); its U k-steps read their operands at constant offsets from the running per-lane
    // addresses, which advance once per row-step.  Fragments of the next k-step are read from LDS while
    // the MFMAs of the current one issue.  The tile count is a compile-time constant per case so that the
    // MFMA block is straight-line code.
    if constexpr (NTL > 0) {
      const int kwg = p.KW / U;
      const int all_rs = (p.cgrps / CG_STEP) * p.KH * kwg;
      const int first = wk * all_rs / WK, nrs = (wk + 1) * all_rs / WK - first;
      if (nrs > 0) {
      int cg = first / (p.KH * kwg), kh = (first - cg * p.KH * kwg) / kwg, kq = first - (cg * p.KH + kh) * kwg;
      // byte strides of the three levels of a row-step index, for A (pixels) and B (weights)
      constexpr int B_TAP = BF ? BN * (KCB + 8) * 2 : 4;   // (bf16: KCB channels per chunk, rows padded by 8)
      const int A_KQ = U * 16, A_KH = p.Wp * 16, A_CG = CG_STEP * cg_stride * 16;
      const int B_KQ = U * B_TAP, B_KH = p.KW * B_TAP, B_CG = BF ? CG_STEP * CI * 2 : CI * KHW * 4;
      int a_addr[NTL], b_addr[TN];
      {
        const int a_off = cg * A_CG + kh * A_KH + kq * A_KQ, b_off = cg * B_CG + kh * B_KH + kq * B_KQ;
#pragma unroll
        for (int t = 0; t < NTL; ++t) a_addr[t] = a_base[t] + a_off;
#pragma unroll
        for (int u = 0; u < TN; ++u) b_addr[u] = b_base[u] + b_off;
      }
      Frag a0[NTL], b0[TN], a1[NTL], b1[TN];
      auto read = [&](auto j_c, Frag (&a)[NTL], Frag (&b)[TN]) {
        constexpr int j = decltype(j_c)::value;
        using Raw = std::conditional_t<BF, uint4, float>;
#pragma unroll
        for (int u = 0; u < TN; ++u)
          b[u] = __builtin_bit_cast(Frag, *reinterpret_cast<const Raw*>(smem + b_addr[u] + j * B_TAP));
#pragma unroll
        for (int t = 0; t < NTL; ++t)
          a[t] = __builtin_bit_cast(Frag, *reinterpret_cast<const Raw*>(smem + a_addr[t] + j * 16));
      };
      auto advance = [&]() {     // wave-uniform deltas, added in place
        int da = A_KQ, db = B_KQ;
        if (++kq == kwg) {
          kq = 0; da += A_KH - kwg * A_KQ; db += B_KH - kwg * B_KQ;
          if (++kh == p.KH) { kh = 0; da += A_CG - p.KH * A_KH; db += B_CG - p.KH * B_KH; }
        }
#pragma unroll
        for (int t = 0; t < NTL; ++t) a_addr[t] += da;
#pragma unroll
        for (int u = 0; u < TN; ++u) b_addr[u] += db;
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
      // k-step j of a row-step whose first k-step's fragments sit in buffer P; NEXT: another row-step follows
      auto kstep = [&](auto j_c, auto p_c, auto next_c) {
        constexpr int j = decltype(j_c)::value;
        constexpr bool cur1 = ((decltype(p_c)::value + j) & 1) != 0;
        auto body = [&](Frag (&ca)[NTL], Frag (&cb)[TN], Frag (&oa)[NTL], Frag (&ob)[TN]) {
          if constexpr (j + 1 < U) {
            read(std::integral_constant<int, (j + 1 < U ? j + 1 : 0)>{}, oa, ob);
          } else if constexpr (decltype(next_c)::value) {
            advance();
            read(std::integral_constant<int, 0>{}, oa, ob);
          }
          mfmas(ca, cb);
          // issue order: one LDS read after each of the first MFMAs, so that the next k-step's fragments
          // are in flight under this k-step's matrix work instead of right before their first use
          if constexpr (j + 1 < U || decltype(next_c)::value) {
            constexpr int NR = NTL + TN, NM = NTL * TN, NP = NR < NM ? NR : NM;
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
        if constexpr (cur1) body(a1, b1, a0, b0);
        else body(a0, b0, a1, b1);
      };
      auto rowstep = [&](auto p_c, auto next_c) {
        kstep(std::integral_constant<int, 0>{}, p_c, next_c);
        if constexpr (U > 1) kstep(std::integral_constant<int, 1>{}, p_c, next_c);
        if constexpr (U > 2) kstep(std::integral_constant<int, 2>{}, p_c, next_c);
        static_assert(U <= 3, "extend the k-steps above");
      };
      // U is odd, so the buffer holding a row-step's first fragments alternates; the steady state is
      // branch-free so that the waits on LDS can be exact
      constexpr std::integral_constant<int, 0> even{};
      constexpr std::integral_constant<int, 1> odd{};
      read(std::integral_constant<int, 0>{}, a0, b0);
      int rs = 0;
      // the first iterations are peeled: each sends one slice of the next chunk's requests first
      auto peeled = [&](auto slice_c) {
        if (more) fetch(ch + 1, slice_c);
        if (rs + 2 < nrs) {
          rowstep(even, std::true_type{});
          rowstep(odd, std::true_type{});
          rs += 2;
        }
      };
      peeled(std::integral_constant<int, 0>{});
      if constexpr (kSlices > 1) peeled(std::integral_constant<int, 1>{});
      if constexpr (kSlices > 2) peeled(std::integral_constant<int, 2>{});
      if constexpr (kSlices > 3) peeled(std::integral_constant<int, 3>{});
      static_assert(kSlices <= 4, "one peeled iteration per slice");
      requested = true;
      for (; rs + 2 < nrs; rs += 2) {
        rowstep(even, std::true_type{});
        rowstep(odd, std::true_type{});
      }
      if (rs + 1 < nrs) { rowstep(even, std::true_type{}); rowstep(odd, std::false_type{}); }
      else rowstep(even, std::false_type{});
      }
    }
    if (more && !requested) fetch(ch + 1, std::integral_constant<int, -1>{});   // (waves without k-steps in this chunk)
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
          for (int u = 0; u < TN; ++u) red[(((wn * WM + wm) * TM + t) * TN + u) * 64 + lane] = acc[t][u];
      }
      __syncthreads();
      if (wk == 0) {
#pragma unroll
        for (int t = 0; t < NTL; ++t)
#pragma unroll
          for (int u = 0; u < TN; ++u) acc[t][u] += red[(((wn * WM + wm) * TM + t) * TN + u) * 64 + lane];
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
        float* op = reinterpret_cast<float*>(out) + (int64_t)ksp * p.split_stride;
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
  if (probe && threadIdx.x == 0) {
    probe[(long long)blockIdx.x * 4 + 2] = wall_clock64();
    probe[(long long)blockIdx.x * 4 + 3] = clock64();
  }
}

constexpr int kMaxLdsBytes = 160 * 1024;   // all of a CU's LDS

struct Variant {
  int WM, WN, WK, TM, TN;
  int XI, WI;    // per thread and chunk: X items (4 pixels x CI channels) and weight pieces
  int KC;        // channels per chunk (fp32 variants may fall back to smaller multiples)
  bool wnat;     // fp32: contiguous weight rows staged in 16-byte pieces
  bool one;      // only for reductions that fit a single chunk (nothing is prefetched during the MFMAs)
  constexpr int NT() const { return WM * WN * WK * 64; }
  constexpr int BN() const { return WN * TN * 16; }
  constexpr int MT() const { return WM * TM; }
};
// Tile variants, 8 waves each.  Row tiles x column tiles per wave, waves along M x N x K:
//   fp32 0-2:  any weight strides, 8 channels per chunk (the backward-data adjoint runs here)
//   fp32 3-8:  forward weight layout [o][c][kh][kw], 16 or 32 channels per chunk (what fits the registers)
//   fp32 9-10: as 4 and 5 with up to 32 channels per chunk (half as many chunk round trips)
//   fp32 11:   64 output channels like 3, half its rows, K split over two waves
//   bf16 0-5:  packed weights, 32 channels per chunk
//   bf16 6:    packed weights, at most 64 channels per group, staged in one go
//   fp32 12:   as 10 for at most 128 pixels per block, up to 64 channels per chunk
//   bf16 7-8:  as 1 and 2 with 64 channels per chunk
//   bf16 9:    as 8 for at most 128 pixels per block, 128 channels per chunk
//   fp32 13:   128 output channels x 256 pixels (4 x 4 tiles per wave): twice the reuse of every staged input pixel,
//              for 1x1 windows (matrix products), where nothing else reuses it
//   bf16 10:   the same for bf16 (packed weights, 64 channels per chunk; 1x1 windows only)
constexpr int kNumF32Variants = 14, kNumBf16Variants = 11;
constexpr Variant kF32Variants[kNumF32Variants] = {
    {4, 2, 1, 7, 2, 1, 9, 8, false}, {4, 2, 1, 7, 1, 1, 5, 8, false}, {8, 1, 1, 4, 1, 1, 3, 8, false},
    {4, 2, 1, 7, 2, 1, 5, 16, true}, {4, 1, 2, 7, 2, 1, 3, 16, true}, {2, 1, 4, 7, 2, 1, 3, 16, true},
    {1, 1, 8, 4, 4, 1, 5, 16, true}, {4, 2, 1, 7, 1, 2, 5, 32, true}, {8, 1, 1, 4, 1, 2, 3, 32, true},
    {4, 1, 2, 7, 2, 1, 5, 32, true}, {2, 1, 4, 7, 2, 1, 5, 32, true}, {2, 2, 2, 7, 2, 1, 5, 16, true},
    {2, 1, 4, 4, 2, 2, 9, 64, true}, {4, 2, 1, 4, 4, 1, 5, 32, true}};
constexpr Variant kBf16Variants[kNumBf16Variants] = {
    {4, 2, 1, 7, 2, 1, 6, 32, false}, {4, 1, 2, 7, 2, 1, 3, 32, false}, {2, 1, 4, 7, 2, 1, 3, 32, false},
    {1, 1, 8, 4, 4, 1, 6, 32, false}, {4, 2, 1, 7, 1, 2, 3, 32, false}, {8, 1, 1, 4, 1, 2, 2, 32, false},
    {4, 2, 1, 7, 2, 4, 11, 64, false, true}, {4, 1, 2, 7, 2, 1, 6, 64, false}, {2, 1, 4, 7, 2, 1, 6, 64, false},
    {2, 1, 4, 4, 2, 2, 10, 128, false}, {4, 2, 1, 4, 4, 1, 3, 64, false}};

template <bool BF, int VI, int U, int WF, bool OUTBF>
void launch_variant(const MfmaParams& p, const void* X, const void* W, void* out, hipStream_t s) {
  constexpr Variant v = BF ? kBf16Variants[VI % kNumBf16Variants] : kF32Variants[VI % kNumF32Variants];
  const int grid = p.n_mblocks * p.n_nblocks * p.G * p.ksplit;
  auto kernel = conv_mfma<BF, v.wnat, v.WM, v.WN, v.WK, v.TM, v.TN, v.XI, v.WI, v.one, (BF ? v.KC : 0), U, WF, OUTBF>;
  static const hipError_t lds_opt_in =      // once per instantiation: allow more than the default 64 KB
      hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
  (void)lds_opt_in;
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(v.NT()), p.lds_bytes, s, p, X, W, out);
}

}  // namespace

// Launchers of the instantiated variants; each lives in a translation unit of its own.
void launch_mfma_f32_lo(int vi, const MfmaParams& p, const void* X, const void* W, void* out, hipStream_t s);    // variants 0-3
void launch_mfma_f32_hi(int vi, const MfmaParams& p, const void* X, const void* W, void* out, hipStream_t s);    // variants 4-13
void launch_mfma_bf16_f32out(int vi, const MfmaParams& p, const void* X, const void* W, void* out, hipStream_t s);
void launch_mfma_bf16_bf16out(int vi, const MfmaParams& p, const void* X, const void* W, void* out, hipStream_t s);

}  // namespace syno
