// The C ABI of include/syno.h: argument checks and dispatch to the kernel families.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdio>
#include <new>
#include <string>
#include <vector>

#include "plan.h"

// A chain owns the plans of its stages.
struct syno_chain {
  std::vector<syno_plan*> stage;
  // Backward-data of stage i writes the gradient that stage i-1 reads as its upstream gradient, so its result
  // type must be stage i-1's input type; where that differs from the stage's own output type (a bf16 stage with an
  // fp32 result) the same graph is planned once more with that result type, for backward-data only (else nullptr).
  std::vector<syno_plan*> bwd_data;
  size_t ws_fwd = 0;        // largest forward workspace of any stage
  size_t ws_bwd_stage = 0;  // largest gradient-call workspace of any stage
  size_t grad_bytes = 0;    // one intermediate-gradient buffer (two are used, alternating)
  // chains written by the materialised-reduction pass: the stage that keeps the graph's weight (-1: every stage
  // has its own); the other stages have none and multiply by the constant one below
  int32_t weight_stage = -1;
  std::vector<int32_t> stage_weight;   // per stage: which of the graph's weights it takes (-1: none)
  ~syno_chain() {
    for (syno_plan* p : stage) delete p;
    for (syno_plan* p : bwd_data) delete p;
  }
};

namespace syno {
syno_status launch_bandwidth(const syno_plan* p, int which, const void* A, const void* B, void* out, void* ws,
                             hipStream_t stream);
syno_status launch_view(const syno_plan* p, int which, const void* A, const void* B, void* out, void* ws,
                        hipStream_t stream);
syno_status launch_window(const syno_plan* p, int which, const void* A, const void* B, void* out, void* ws,
                          hipStream_t stream);
syno_status launch_mfma(const syno_plan* p, int which, const void* A, const void* B, void* out, void* ws,
                        hipStream_t stream);
std::string mfma_describe(const syno_plan* p, int which);
syno_status launch_mfma_dw(const syno_plan* p, const void* A, const void* B, void* out, void* ws, hipStream_t stream);
std::string mfma_dw_describe(const syno_plan* p);
}

// The value 1 in both element types, for stages without a weight: fp32 in word 0, bf16 in the low half of word 1.
static __device__ __align__(16) uint32_t g_unit_words[4] = {0x3F800000u, 0x00003F80u, 0u, 0u};

// Scratch memory of syno_backward_weight_static: one copy per GPU, held until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress; kernels get the per-device address looked up below.
static __device__ __align__(256) unsigned char scratch[SYNO_STATIC_SCRATCH_BYTES];

namespace {

// Device address of `scratch` on the current device, looked up once per device with that device current.
void* static_scratch() {
  constexpr int kMaxDevices = 64;
  static std::atomic<void*> cache[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = cache[dev].load(std::memory_order_acquire);
  if (!p) {
    void* sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return nullptr;
    p = sym;
    cache[dev].store(p, std::memory_order_release);
  }
  return p;
}

// Device address of the constant one in element type `t` on the current device (each device has its own copy of
// the array; the address is looked up once per device).
const void* unit_weight(syno_dtype t) {
  constexpr int kMaxDevices = 64;
  static std::atomic<char*> cache[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  char* p = cache[dev].load(std::memory_order_acquire);
  if (!p) {
    void* sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(g_unit_words)) != hipSuccess || !sym) return nullptr;
    p = static_cast<char*>(sym);
    cache[dev].store(p, std::memory_order_release);
  }
  return t == SYNO_BF16 ? p + 4 : p;
}

const char* const kKernelNames[syno::KERNEL_COUNT] = {
    "generic_index_program", "bandwidth_depthwise", "bandwidth_share_window", "bandwidth_view", "mfma_contraction_f32", "mfma_contraction_bf16",
    "mfma_contraction_transposed", "mfma_contraction_phases"};

syno_status run(const syno_plan* plan, int which, const void* A, const void* B, void* out, void* ws,
                hipStream_t stream) {
  if (!plan || !A || !B || !out) return SYNO_ERR_NULL;
  const syno::Launch& L = plan->launch[which];
  if (L.workspace && !ws) return SYNO_ERR_WORKSPACE;
  switch (L.kernel) {
    case syno::KERNEL_GENERIC: return syno::launch_generic(plan, which, A, B, out, stream);
    case syno::KERNEL_BW_DEPTHWISE: return syno::launch_bandwidth(plan, which, A, B, out, ws, stream);
    case syno::KERNEL_BW_WINDOW: return syno::launch_window(plan, which, A, B, out, ws, stream);
    case syno::KERNEL_BW_VIEW: return syno::launch_view(plan, which, A, B, out, ws, stream);
    case syno::KERNEL_MFMA_F32:
    case syno::KERNEL_MFMA_BF16:
      if (which == SYNO_BWD_WEIGHT) return syno::launch_mfma_dw(plan, A, B, out, ws, stream);
      return syno::launch_mfma(plan, which, A, B, out, ws, stream);
    case syno::KERNEL_MFMA_TRANSPOSED:
      // forward: the weight is the image and the input the filter; the gradients keep their operand order
      // (upstream gradient first) and only name the other contraction of the inner plan
      if (which == SYNO_FWD) return run(plan->inner, SYNO_FWD, B, A, out, ws, stream);
      if (L.variant == syno::kViaTransposedCopy) {
        // dX = G * W^T as a product of its own: W^T goes into the head of the workspace and is the "image" of that
        // product's 1x1 convolution, G its filter
        const int64_t K = plan->w_shape[0], N = plan->w_shape[1];
        const int esz = plan->in_dtype == SYNO_BF16 ? 2 : 4;
        const syno_status st = syno::launch_transpose_2d(B, ws, K, N, esz, stream);
        if (st != SYNO_OK) return st;
        const size_t head = ((size_t)K * N * esz + 255) & ~(size_t)255;
        return run(plan->inner_dx, SYNO_FWD, ws, A, out, static_cast<char*>(ws) + head, stream);
      }
      return run(plan->inner, L.variant, A, B, out, ws, stream);
    case syno::KERNEL_MFMA_PHASES: {
      // gradients of a strided convolution on the stride's phase planes (see the planner)
      if (!ws) return SYNO_ERR_WORKSPACE;
      const syno::ConvLike& c = plan->conv;
      const int window = plan->phase_window;
      const size_t esz = plan->in_dtype == SYNO_BF16 ? 2 : 4, osz = plan->out_dtype == SYNO_BF16 ? 2 : 4;
      const int ps = plan->phase_s;
      const size_t CP = (size_t)c.Cg * ps * ps;
      auto round_up = [](size_t n) { return (n + 255) & ~(size_t)255; };
      char* w0 = static_cast<char*>(ws);
      if (which == SYNO_BWD_WEIGHT) {          // A = G, B = X, out = dW
        void* Xp = w0;
        float* dWp = reinterpret_cast<float*>(w0 + round_up((size_t)plan->phase_view_x->out_elems * esz));
        void* rest = reinterpret_cast<char*>(dWp) + round_up((size_t)c.Og * CP * window * window * 4);
        const void* one = unit_weight(plan->in_dtype);
        if (!one) return SYNO_ERR_HIP;
        syno_status st = run(plan->phase_view_x, SYNO_FWD, B, one, Xp, nullptr, stream);
        if (st != SYNO_OK) return st;
        st = run(plan->phase_conv_dw, SYNO_BWD_WEIGHT, A, Xp, dWp, rest, stream);
        if (st != SYNO_OK) return st;
        return syno::launch_phase_weight_gather(c, ps, window, dWp, static_cast<float*>(out), stream);
      }
      // A = G, B = W, out = dX
      void* Wpp = w0;
      void* dXp = w0 + round_up(CP * c.Og * window * window * esz);
      void* rest = static_cast<char*>(dXp) + round_up((size_t)plan->phase_view_dx->out_elems * osz);
      const void* one = unit_weight(plan->out_dtype);
      if (!one) return SYNO_ERR_HIP;
      syno_status st = syno::launch_phase_weight_build(c, ps, window, (int)esz, B, Wpp, stream);
      if (st != SYNO_OK) return st;
      st = run(plan->phase_conv_dx, SYNO_FWD, A, Wpp, dXp, rest, stream);
      if (st != SYNO_OK) return st;
      void* view_ws = static_cast<char*>(rest) + plan->phase_conv_dx->launch[SYNO_FWD].workspace;
      return run(plan->phase_view_dx, SYNO_BWD_DATA, dXp, one, out, view_ws, stream);
    }
    default: return SYNO_ERR_UNSUPPORTED;
  }
}
}  // namespace

extern "C" {

syno_status syno_plan_create(const syno_desc* desc, syno_plan** plan) {
  if (!desc || !plan) return SYNO_ERR_NULL;
  *plan = nullptr;
  syno_plan* p = nullptr;
  try {     // (the planner's containers may throw; nothing may cross this boundary)
    p = new syno_plan();
    std::string why;
    const syno_status st = syno::build_plan(desc, p, &why);
    if (st != SYNO_OK) {
      delete p;
      return st;
    }
  } catch (...) {
    delete p;
    return SYNO_ERR_UNSUPPORTED;
  }
  *plan = p;
  return SYNO_OK;
}

syno_status syno_plan_destroy(syno_plan* plan) {
  delete plan;
  return SYNO_OK;
}

syno_status syno_forward(const syno_plan* plan, const void* X, const void* W, void* out, void* ws,
                         hipStream_t stream) {
  return run(plan, SYNO_FWD, X, W, out, ws, stream);
}

syno_status syno_backward_data(const syno_plan* plan, const void* G, const void* W, void* dX, void* ws,
                               hipStream_t stream) {
  return run(plan, SYNO_BWD_DATA, G, W, dX, ws, stream);
}

syno_status syno_backward_weight(const syno_plan* plan, const void* X, const void* G, void* dW, void* ws,
                                 hipStream_t stream) {
  // the lowered forms take the upstream gradient first
  return run(plan, SYNO_BWD_WEIGHT, G, X, dW, ws, stream);
}

syno_status syno_backward_weight_static(const syno_plan* plan, const void* X, const void* G, void* dW,
                                        hipStream_t stream) {
  if (!plan || !X || !G || !dW) return SYNO_ERR_NULL;
  const size_t need = plan->launch[SYNO_BWD_WEIGHT].workspace;
  if (need > SYNO_STATIC_SCRATCH_BYTES) return SYNO_ERR_SCRATCH;
  void* ws = nullptr;
  if (need) {
    ws = static_scratch();
    if (!ws) return SYNO_ERR_HIP;
  }
  // (every kernel writes the part of the scratch it later reads, so nothing has to be cleared between calls)
  return run(plan, SYNO_BWD_WEIGHT, G, X, dW, ws, stream);
}

syno_status syno_plan_workspace_bytes(const syno_plan* plan, int which, size_t* bytes) {
  if (!plan || !bytes) return SYNO_ERR_NULL;
  if (which < 0 || which > 2) return SYNO_ERR_SHAPE;
  *bytes = plan->launch[which].workspace;
  return SYNO_OK;
}

syno_status syno_plan_shapes(const syno_plan* plan, int32_t* x_rank, int64_t* x_shape, int32_t* w_rank,
                             int64_t* w_shape, int32_t* out_rank, int64_t* out_shape) {
  if (!plan || !x_rank || !x_shape || !w_rank || !w_shape || !out_rank || !out_shape) return SYNO_ERR_NULL;
  *x_rank = plan->x_rank;
  *w_rank = plan->w_rank;
  *out_rank = plan->out_rank;
  for (int i = 0; i < plan->x_rank; ++i) x_shape[i] = plan->x_shape[i];
  for (int i = 0; i < plan->w_rank; ++i) w_shape[i] = plan->w_shape[i];
  for (int i = 0; i < plan->out_rank; ++i) out_shape[i] = plan->out_shape[i];
  return SYNO_OK;
}

const char* syno_plan_kernel(const syno_plan* plan, int which) {
  if (!plan || which < 0 || which > 2) return nullptr;
  return kKernelNames[plan->launch[which].kernel];
}

syno_status syno_plan_describe(const syno_plan* plan, int which, char* buf, size_t size) {
  if (!plan || !buf) return SYNO_ERR_NULL;
  if (which < 0 || which > 2 || size == 0) return SYNO_ERR_SHAPE;
  std::string d = kKernelNames[plan->launch[which].kernel];
  switch (plan->launch[which].kernel) {
    case syno::KERNEL_GENERIC: d += plan->launch[which].coop ? " workgroup-per-target" : " lane-per-target"; break;
    case syno::KERNEL_MFMA_F32:
    case syno::KERNEL_MFMA_BF16:
      d += " " + (which == SYNO_BWD_WEIGHT ? syno::mfma_dw_describe(plan) : syno::mfma_describe(plan, which));
      break;
    case syno::KERNEL_BW_VIEW: d += " " + syno::view_describe(plan, which); break;
    case syno::KERNEL_MFMA_PHASES: {
      char inner[400];
      const syno_plan* conv = which == SYNO_BWD_WEIGHT ? plan->phase_conv_dw : plan->phase_conv_dx;
      if (syno_plan_describe(conv, which == SYNO_BWD_WEIGHT ? SYNO_BWD_WEIGHT : SYNO_FWD, inner, sizeof(inner)) == SYNO_OK)
        d += std::string(which == SYNO_BWD_WEIGHT ? " space-to-depth of X, then the weight gradient of a stride-1 convolution over the phase planes: "
                                                  : " forward contraction onto the phase planes of dX, then depth-to-space: ") + inner;
      break;
    }
    case syno::KERNEL_MFMA_TRANSPOSED: {
      char inner[400];
      if (plan->launch[which].variant == syno::kViaTransposedCopy) {
        if (syno_plan_describe(plan->inner_dx, SYNO_FWD, inner, sizeof(inner)) == SYNO_OK)
          d += std::string(" as the product G * W^T (transposed copy of W), a 1x1 convolution: ") + inner;
      } else if (syno_plan_describe(plan->inner, plan->launch[which].variant, inner, sizeof(inner)) == SYNO_OK)
        d += std::string(" as 1x1 convolution: ") + inner;
      break;
    }
    default: break;
  }
  snprintf(buf, size, "%s", d.c_str());
  return SYNO_OK;
}

syno_status syno_plan_free_size(const syno_plan* plan, int which, int64_t* free_size) {
  if (!plan || !free_size) return SYNO_ERR_NULL;
  if (which < 0 || which > 2) return SYNO_ERR_SHAPE;
  *free_size = plan->prog[which].n_free;
  return SYNO_OK;
}

syno_status syno_debug_gather(const syno_plan* plan, int which, const int64_t* t_flat, const int64_t* q_flat,
                              int64_t n, int32_t* a_off, int32_t* b_off, hipStream_t stream) {
  if (!plan || (n > 0 && (!t_flat || !q_flat || !a_off || !b_off))) return SYNO_ERR_NULL;
  if (which < 0 || which > 2 || n < 0) return SYNO_ERR_SHAPE;
  return syno::launch_debug_gather(plan, which, t_flat, q_flat, n, a_off, b_off, stream);
}

syno_status syno_debug_gather_host(const syno_plan* plan, int which, const int64_t* t_flat, const int64_t* q_flat,
                                   int64_t n, int32_t* a_off, int32_t* b_off) {
  if (!plan || (n > 0 && (!t_flat || !q_flat || !a_off || !b_off))) return SYNO_ERR_NULL;
  if (which < 0 || which > 2 || n < 0) return SYNO_ERR_SHAPE;
  return syno::host_debug_gather(plan, which, t_flat, q_flat, n, a_off, b_off);
}

namespace {
// Plans every stage.  dx_dtype: element type of the chain's dX (-1: the first stage's own output type).
syno_status chain_create(const syno_desc* stages, int32_t n_stages, int dx_dtype, syno_chain** chain) {
  if (n_stages < 1 || n_stages > 8) return SYNO_ERR_SHAPE;
  syno_chain* c = new syno_chain();
  const auto esize = [](syno_dtype t) { return t == SYNO_BF16 ? size_t(2) : size_t(4); };
  const auto fail = [&](syno_status st) { delete c; return st; };
  for (int i = 0; i < n_stages; ++i) {
    syno_plan* p = nullptr;
    syno_status st = syno_plan_create(&stages[i], &p);
    if (st != SYNO_OK) return fail(st);
    c->stage.push_back(p);
    c->bwd_data.push_back(nullptr);
    if (i > 0) {
      const syno_plan* q = c->stage[i - 1];
      if (q->out_elems != p->x_elems || q->out_dtype != p->in_dtype) return fail(SYNO_ERR_SHAPE);
    }
    // the type this stage's backward-data must produce
    const syno_dtype want = i > 0 ? c->stage[i - 1]->in_dtype : (dx_dtype < 0 ? p->out_dtype : (syno_dtype)dx_dtype);
    if (want != p->out_dtype) {
      syno_desc d = stages[i];
      d.out_dtype = want;
      st = syno_plan_create(&d, &c->bwd_data[i]);
      if (st != SYNO_OK) return fail(st);
    }
    const syno_plan* pb = c->bwd_data[i] ? c->bwd_data[i] : p;
    c->ws_fwd = std::max(c->ws_fwd, p->launch[SYNO_FWD].workspace);
    c->ws_bwd_stage = std::max(c->ws_bwd_stage, std::max(pb->launch[SYNO_BWD_DATA].workspace, p->launch[SYNO_BWD_WEIGHT].workspace));
    if (i > 0) c->grad_bytes = std::max(c->grad_bytes, ((size_t(p->x_elems) * esize(want)) + 255) & ~size_t(255));
  }
  *chain = c;
  return SYNO_OK;
}
}  // namespace

syno_status syno_chain_create_materialized(const syno_desc* desc, syno_chain** chain) {
  if (!desc || !chain) return SYNO_ERR_NULL;
  *chain = nullptr;
  try {
    std::vector<syno::OwnedDesc> stages;
    std::vector<int32_t> stage_weight;
    syno_status st = syno::materialise(desc, stages, stage_weight);
    if (st != SYNO_OK) return st;
    std::vector<syno_desc> views;
    for (const syno::OwnedDesc& o : stages) views.push_back(o.view());
    // dX of the whole graph has the graph's output type, whatever type the first stage stores its result in
    st = chain_create(views.data(), (int32_t)views.size(), (int)desc->out_dtype, chain);
    if (st == SYNO_OK) {
      (*chain)->stage_weight = stage_weight;
      (*chain)->weight_stage = -1;
      for (size_t i = 0; i < stage_weight.size(); ++i)
        if (stage_weight[i] == 0) (*chain)->weight_stage = (int32_t)i;
    }
    return st;
  } catch (...) {
    return SYNO_ERR_UNSUPPORTED;
  }
}

int32_t syno_chain_weight_stage(const syno_chain* chain) { return chain ? chain->weight_stage : -1; }

int32_t syno_chain_stage_weight(const syno_chain* chain, int32_t stage) {
  if (!chain || stage < 0 || stage >= (int32_t)chain->stage.size()) return -1;
  return chain->stage_weight.empty() ? stage : chain->stage_weight[(size_t)stage];
}

syno_status syno_chain_create(const syno_desc* stages, int32_t n_stages, syno_chain** chain) {
  if (!stages || !chain) return SYNO_ERR_NULL;
  *chain = nullptr;
  try {
    return chain_create(stages, n_stages, -1, chain);
  } catch (...) {
    return SYNO_ERR_UNSUPPORTED;
  }
}

syno_status syno_chain_destroy(syno_chain* chain) {
  delete chain;
  return SYNO_OK;
}

int32_t syno_chain_stages(const syno_chain* chain) { return chain ? int32_t(chain->stage.size()) : 0; }

const syno_plan* syno_chain_plan(const syno_chain* chain, int32_t stage) {
  if (!chain || stage < 0 || stage >= int32_t(chain->stage.size())) return nullptr;
  return chain->stage[size_t(stage)];
}

syno_status syno_chain_workspace_bytes(const syno_chain* chain, int which, size_t* bytes) {
  if (!chain || !bytes) return SYNO_ERR_NULL;
  if (which < 0 || which > 1) return SYNO_ERR_SHAPE;
  const size_t ws_stage = (chain->ws_bwd_stage + 255) & ~size_t(255);
  *bytes = which == 0 ? chain->ws_fwd : ws_stage + 2 * chain->grad_bytes;
  return SYNO_OK;
}

syno_status syno_chain_forward(const syno_chain* chain, const void* X, const void* const* W, void* const* act,
                               void* out, void* workspace, hipStream_t stream) {
  if (!chain || !X || !W || !out) return SYNO_ERR_NULL;
  const size_t n = chain->stage.size();
  if (n > 1 && !act) return SYNO_ERR_NULL;
  if (chain->ws_fwd && !workspace) return SYNO_ERR_WORKSPACE;
  const void* cur = X;
  for (size_t i = 0; i < n; ++i) {
    void* dst = i + 1 < n ? act[i] : out;
    const bool own = chain->stage_weight.empty() || chain->stage_weight[i] >= 0;
    const void* Wi = own ? W[i] : unit_weight(chain->stage[i]->in_dtype);
    if (!Wi) return own ? SYNO_ERR_NULL : SYNO_ERR_HIP;
    const syno_status st = run(chain->stage[i], SYNO_FWD, cur, Wi, dst, workspace, stream);
    if (st != SYNO_OK) return st;
    cur = dst;
  }
  return SYNO_OK;
}

syno_status syno_chain_backward(const syno_chain* chain, const void* X, const void* const* W,
                                const void* const* act, const void* G, void* dX, void* const* dW,
                                void* workspace, hipStream_t stream) {
  if (!chain || !X || !W || !G || !dW) return SYNO_ERR_NULL;
  const size_t n = chain->stage.size();
  if (n > 1 && !act) return SYNO_ERR_NULL;
  size_t need = 0;
  syno_chain_workspace_bytes(chain, 1, &need);
  if (need && !workspace) return SYNO_ERR_WORKSPACE;
  // workspace: [stage workspace | gradient buffer 0 | gradient buffer 1]
  char* const base = static_cast<char*>(workspace);
  char* const grad0 = base + ((chain->ws_bwd_stage + 255) & ~size_t(255));
  const void* g = G;
  for (size_t i = n; i-- > 0;) {
    const void* in = i == 0 ? X : act[i - 1];
    const bool own = chain->stage_weight.empty() || chain->stage_weight[i] >= 0;
    const void* Wi = own ? W[i] : unit_weight(chain->stage[i]->in_dtype);
    if (!Wi) return own ? SYNO_ERR_NULL : SYNO_ERR_HIP;
    syno_status st = SYNO_OK;
    if (own) {     // a stage without a weight has no weight gradient
      if (!dW[i]) return SYNO_ERR_NULL;
      st = run(chain->stage[i], SYNO_BWD_WEIGHT, g, in, dW[i], base, stream);
      if (st != SYNO_OK) return st;
    }
    void* dst = i == 0 ? dX : static_cast<void*>(grad0 + (i & 1) * chain->grad_bytes);
    if (!dst) break;   // first stage and the caller does not want dX
    st = run(chain->bwd_data[i] ? chain->bwd_data[i] : chain->stage[i], SYNO_BWD_DATA, g, Wi, dst, base, stream);
    if (st != SYNO_OK) return st;
    g = dst;
  }
  return SYNO_OK;
}

const char* syno_status_string(syno_status s) {
  switch (s) {
    case SYNO_OK: return "ok";
    case SYNO_ERR_NULL: return "null pointer";
    case SYNO_ERR_INVALID_DESC: return "invalid primitive graph";
    case SYNO_ERR_SHAPE: return "argument out of range";
    case SYNO_ERR_UNSUPPORTED: return "unsupported";
    case SYNO_ERR_WORKSPACE: return "workspace required";
    case SYNO_ERR_HIP: return "HIP runtime error";
    case SYNO_ERR_SCRATCH: return "the call needs more scratch memory than the library's static buffer holds";
  }
  return "unknown status";
}

}  // extern "C"
