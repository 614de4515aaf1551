// Internal: lowered forms a plan holds, shared by the planner (host) and the kernels.
#pragma once
#include <stdint.h>
#include <string>
#include <vector>

#include "syno.h"

namespace syno {

constexpr int kMaxSlots = 24;   // distinct coordinate values (Share copies alias one slot)
constexpr int kMaxOps = 32;
constexpr int kMaxAxes = 8;

// ---------------------------------------------------------------------------------------------
// Index program: the general lowered form of one contraction.  A target element (decoded from
// its flat index along `tgt`) and a free point (decoded along `fre`) fill some slots; the ops
// then derive every other coordinate, forwards (Table 1 as written) or inverted (for the
// gradients), and the two source offsets are dot products of slots with strides.
// ---------------------------------------------------------------------------------------------
enum OpKind : int32_t {
  OP_MULADD = 0,   // v[d0] = v[a]*p0 + v[b]                       Split forwards, Merge inverted
  OP_DIVMOD = 1,   // v[d0] = v[a]/p0 ; v[d1] = v[a]%p0            Merge forwards, Split inverted  (p1 = division_magic(p0))
  OP_SHIFT  = 2,   // v[d0] = (v[a] + p1 + p2*v[b]) mod p0, >= 0   Shift, either way
  OP_ADDCHK = 3,   // t = v[a] + p2*v[b] + p1 ; ok &= 0<=t<p0 ; v[d0]=t   Unfold, either way
  OP_MUL    = 4,   // v[d0] = v[a]*p0                              Stride forwards
  OP_DIVCHK = 5    // ok &= v[a]%p0==0 ; v[d0] = v[a]/p0           Stride inverted                 (p1 = division_magic(p0))
};

struct IndexOp {
  int32_t kind, a, b, d0, d1, p0, p1, p2;
};

struct AxisRef {
  int32_t slot, size, stride;   // target and free axes carry division_magic(size) in `stride` (they have no stride)
};

// Division of a 31-bit unsigned n by a runtime d >= 2 as one high multiplication and a shift:
// n / d == mulhi(n, M) >> s with s = ceil(log2 d) - 1 and M = ceil(2^(32+s) / d), exact for n < 2^31
// (M < 2^32 because d > 2^s; the error M*d - 2^(32+s) < d <= 2^(s+1) stays below one unit at that range).
inline uint32_t division_magic(int64_t d) {
  if (d < 2) return 0;
  int s = 0;
  while ((int64_t(1) << (s + 1)) < d) ++s;
  const uint64_t num = uint64_t(1) << (32 + s);     // s <= 30
  return (uint32_t)((num + (uint64_t)d - 1) / (uint64_t)d);
}

struct IndexProgram {
  int32_t n_tgt, n_fre, n_ops0, n_ops, n_a, n_b;   // ops[0..n_ops0) depend on the target only
  AxisRef tgt[kMaxAxes];     // target tensor axes, outermost first (stride unused)
  AxisRef fre[kMaxAxes];     // free coordinates, outermost first (stride unused)
  IndexOp ops[kMaxOps];
  AxisRef a[kMaxAxes];       // first source: slots and element strides
  AxisRef b[kMaxAxes];       // second source
  int64_t n_target, n_free;  // products of the sizes above
};

// ---------------------------------------------------------------------------------------------
// Convolution-like lowered form: what the forward index map looks like when every X axis is an
// affine function of the iterators, optionally wrapped (Shift) or range-checked (Unfold), on a
// 4-axis input [batch, channel, row, column].  The tuned kernels take this record.
//   out[n, g*Og+o, h, w] = sum_{c,kh,kw} X[n, g*Cg+c, row(h,kh,g), col(w,kw,g)] * W[g,o,c,kh,kw]
//   row = sh*h + kh - ph (+ shift, mod Hi when h_wrap), dropped when outside [0,Hi) otherwise
// ---------------------------------------------------------------------------------------------
struct ConvLike {
  int32_t N, G, Og, Cg, Ho, Wo, Hi, Wi, KH, KW;
  int32_t sh, sw, ph, pw;
  int32_t h_wrap, w_wrap;           // 1: cyclic (mod Hi / Wi), 0: zero outside
  int32_t h_shift, h_shift_g;       // row offset = h_shift + h_shift_g * g (only when wrapped)
  int32_t w_shift, w_shift_g;
  // weight element strides per role (0 when the role has size 1 or is absent)
  int32_t ws_g, ws_o, ws_c, ws_kh, ws_kw;
};

// ---------------------------------------------------------------------------------------------
// Window whose iterator is Shared with the weight but not Reduced (first stage of Operator 1, Fig. 7):
//   out[n,d,g,k,h,w] = sum_c X[n, g*Cg+c, h, w+k-pw] * W[d,g,c,k]      (zero outside the row), pw = K/2
// ---------------------------------------------------------------------------------------------
struct ShareWindow {
  int32_t N, D, G, K, H, W, Cg, pw;
  int32_t ws_d, ws_g, ws_c, ws_k;   // weight element strides per role (0 when the role has size 1)
};

// ---------------------------------------------------------------------------------------------
// Separable gather (no Unfold): every X axis and every W axis is an affine function of digits of the output
// iterators and of the Reduce iterators, optionally wrapped (Shift) when all its digits come from one iterator.
// The two source offsets are then sums of one table per iterator, offX(o,r) = sum_i tabX_i[o_i] + sum_j tabX_j[r_j];
// the kernel builds the tables in LDS from this record.  Without Reduce it is a pure view; with a few sum points
// per output (block sums, small pools) a gather-and-add.
//   group  = one tensor axis: value = sum of its terms + c, taken mod `wrap` when wrap > 0, times `stride`
//   term   = coef * ((o_axis / div) % size), a digit of output axis `axis`
// ---------------------------------------------------------------------------------------------
struct ViewTerm { int32_t group, axis, div, size, coef; };
struct ViewGroup { int32_t tensor, stride, c, wrap, axis; };   // tensor: 0 = X, 1 = W; axis: the one a wrapped or constant group is charged to
constexpr int kMaxViewTerms = 24, kMaxViewGroups = 16;
struct ViewStream {
  int32_t n_axes, n_terms, n_groups;
  int32_t n_red;                 // Reduce iterators: axes n_axes .. n_axes+n_red-1 of `size` (few sum points per output)
  int32_t size[2 * kMaxAxes];
  ViewTerm term[kMaxViewTerms];
  ViewGroup group[kMaxViewGroups];
  int32_t one_to_one;            // no Reduce and only Split, Merge, Shift and Share: every X element is read by exactly one output
};

enum KernelId : int32_t {
  KERNEL_GENERIC = 0,
  KERNEL_BW_DEPTHWISE,
  KERNEL_BW_WINDOW,
  KERNEL_BW_VIEW,
  KERNEL_MFMA_F32,
  KERNEL_MFMA_BF16,
  KERNEL_MFMA_TRANSPOSED,   // a matrix product run as the 1x1 convolution with exchanged operand roles (plan->inner)
  KERNEL_MFMA_PHASES,       // gradients of a strided convolution through the stride's phase planes (plan->phase_*)
  KERNEL_COUNT
};

struct Launch {
  KernelId kernel = KERNEL_GENERIC;
  int32_t coop = 0;           // generic kernel: one workgroup per target (1) or one lane per target (0)
  int32_t variant = 0;        // tile configuration index within the family
  size_t workspace = 0;
  // the family's kernel parameter record, filled when the plan is configured so that a launch only copies it
  alignas(8) unsigned char params[1536] = {};
  bool params_ready = false;
};

}  // namespace syno

struct syno_plan {
  // shapes
  int32_t x_rank = 0, w_rank = 0, out_rank = 0;
  int64_t x_shape[syno::kMaxAxes] = {}, w_shape[syno::kMaxAxes] = {}, out_shape[syno::kMaxAxes] = {};
  int64_t x_elems = 0, w_elems = 0, out_elems = 0, n_reduce = 0;
  syno_dtype in_dtype = SYNO_F32, out_dtype = SYNO_F32;
  syno_plan_options opt{};      // the descriptor's overrides (all 0: the planner decides)
  // lowered forms
  syno::IndexProgram prog[3];
  bool conv_like = false;
  syno::ConvLike conv{};
  bool share_window = false;
  syno::ShareWindow window{};
  syno::Launch launch[3];
  // matrix products: the plan of the equivalent 1x1 convolution (owned); Launch::variant holds its contraction
  syno_plan* inner = nullptr;
  // matrix products: dX = G * W^T is a matrix product too; the plan of ITS 1x1 convolution (owned), whose forward
  // contraction runs on a transposed copy of W in the workspace (Launch::variant = kViaTransposedCopy)
  syno_plan* inner_dx = nullptr;
  // strided convolutions (stride s below the window): the gradients run at stride 1 on the s*s phase planes
  // X[.., s*h'+a, s*w'+b] taken as s*s*C channels.  phase_view_x / phase_view_dx: the space-to-depth view in the input
  // and in the result element type; phase_conv_dw / phase_conv_dx: the stride-1 convolutions whose backward-weight and
  // forward contractions do the work (owned)
  syno_plan *phase_view_x = nullptr, *phase_view_dx = nullptr, *phase_conv_dw = nullptr, *phase_conv_dx = nullptr;
  int32_t phase_window = 0;      // window of those convolutions: 3 (pad 1) or 1
  int32_t phase_s = 0;           // phases per image axis that take part: s, or 1 for a 1x1 window, which only reads phase
                                 // (0, 0) - the view is then the sub-sampling X[.., s*h', s*w'] itself
  ~syno_plan() { delete inner; delete inner_dx; delete phase_view_x; delete phase_view_dx; delete phase_conv_dw; delete phase_conv_dx; }
  bool pure_view = false;
  syno::ViewStream view{};
};

namespace syno {

// A descriptor that owns its arrays (the stages the materialised-reduction pass writes).
struct OwnedDesc {
  std::vector<syno_dim> dims;
  std::vector<syno_prim> prims;
  std::vector<int32_t> xin, win;
  std::vector<int32_t> more_ranks, more_flat;   // further weights, as in syno_desc
  std::vector<int32_t> weight_ids;              // which of the original graph's weights `win` and the further ones are
  syno_dtype in_dtype = SYNO_F32, out_dtype = SYNO_F32;
  syno_plan_options opt{};
  bool has_opt = false;
  // (the returned descriptor points into this object)
  syno_desc view() const {
    syno_desc d{};
    d.n_out = (int32_t)dims.size(); d.out_dims = dims.data();
    d.n_prim = (int32_t)prims.size(); d.prims = prims.data();
    d.n_in = (int32_t)xin.size(); d.input_coords = xin.data();
    d.n_w = (int32_t)win.size(); d.weight_coords = win.data();
    d.in_dtype = in_dtype; d.out_dtype = out_dtype;
    d.options = has_opt ? &opt : nullptr;
    d.n_more_weights = (int32_t)more_ranks.size(); d.more_weight_ranks = more_ranks.data(); d.more_weight_coords = more_flat.data();
    return d;
  }
};

// planner.cpp
// Materialised reduction: cuts `desc` into stages (one stage when no cut lowers the count of multiply-adds);
// stage_weight[i] = which of the graph's weights stage i keeps (-1: none).
syno_status materialise(const syno_desc* desc, std::vector<OwnedDesc>& stages, std::vector<int32_t>& stage_weight);
syno_status build_plan(const syno_desc* desc, syno_plan* plan, std::string* why);

// kernels_generic.hip
syno_status launch_generic(const syno_plan* p, int which, const void* A, const void* B, void* out,
                           hipStream_t stream);
syno_status launch_debug_gather(const syno_plan* p, int which, const int64_t* t, const int64_t* q, int64_t n,
                                int32_t* a_off, int32_t* b_off, hipStream_t stream);
syno_status host_debug_gather(const syno_plan* p, int which, const int64_t* t, const int64_t* q, int64_t n,
                              int32_t* a_off, int32_t* b_off);

// kernels_bandwidth.hip / kernels_mfma.hip: can the family take contraction `which` of this plan?
bool bandwidth_supports(const syno_plan* p, int which);
bool mfma_supports(const syno_plan* p, int which);
// fills launch[which] (tile variant, workspace bytes) for the MFMA family
void mfma_configure(syno_plan* p, int which);
void bandwidth_configure(syno_plan* p, int which);   // fills launch[which].params and .workspace
// kernels_view.hip: separable gathers; view_configure fills launch[which].params
bool view_supports(const syno_plan* p, int which);
void view_configure(syno_plan* p, int which);
std::string view_describe(const syno_plan* p, int which);
// kernels_window.hip: the unreduced-window member of the bandwidth family
bool window_supports(const syno_plan* p, int which);
void window_configure(syno_plan* p, int which);      // fills launch[which].params and .workspace
// conv_rows_bf16.hip: the row-streaming member of the MFMA family (bf16, whole reduction in LDS)
bool rows_supports(const syno_plan* p, int which);
bool rows_configure(syno_plan* p, int which);
std::string rows_describe(const syno_plan* p, int which);
syno_status launch_rows(const syno_plan* p, int which, const void* A, const void* B, void* out, void* ws, hipStream_t stream);
// kernels_mfma.hip: dst[c][r] = src[r][c] for a row-major rows x cols matrix of 2- or 4-byte elements
constexpr int kViaTransposedCopy = 100;
syno_status launch_transpose_2d(const void* src, void* dst, int64_t rows, int64_t cols, int elem_bytes, hipStream_t stream);
// kernels_mfma.hip, gradients of a strided convolution through the phase planes:
// (s = the phases per axis that take part: the stride, or 1 when only phase (0,0) is read)
// dW[o,c,kh,kw] (any strides) = dWp[o][(c*s+a)*s+b][th][tw] with s*dh+a = kh-p, th = dh+1 (window 3) or 0 (window 1)
syno_status launch_phase_weight_gather(const ConvLike& c, int s, int window, const float* dWp, float* dW, hipStream_t stream);
// Wpp[(c*s+a)*s+b][o][th][tw] (contiguous, 2- or 4-byte elements) = W[o,c,kh,kw] with kh = a+p-s*dh, or 0 where there is none
syno_status launch_phase_weight_build(const ConvLike& c, int s, int window, int elem_bytes, const void* W, void* Wpp, hipStream_t stream);
// kernels_mfma_dw.hip: the backward-weight member of the MFMA family
bool mfma_dw_supports(const syno_plan* p);
void mfma_dw_configure(syno_plan* p);

}  // namespace syno
