/*
 * syno.h - C ABI of the MI355X executor for synthesized operators.
 *
 * An operator is a primitive graph (pGraph; paper section 5.1, Fig. 2): the output
 * iterators form the bottom, each primitive of Table 1 rewrites bottom coordinates into top
 * coordinates, and the top coordinates index one data input X and one weight W (the weight
 * receives one copy of every Shared coordinate plus the iterators matched to it, section
 * 5.3).  Each Reduce adds a sum loop, so the operator is the index-mapped contraction
 *
 *     out[o] = sum_r  X[f(o,r)] * W[g(o,r)]                      (Listing 1's loop-nest form)
 *
 * with terms dropped where an Unfold leaves its domain (zero padding).  The library builds a
 * plan from such a graph on concrete sizes (section 5.4: symbols are replaced by sizes
 * before code generation) and evaluates the forward pass and the two gradient contractions
 * of L = sum_o out[o]*G[o] on the GPU.
 *
 * All tensor pointers are DEVICE pointers to dense row-major arrays, 16-byte aligned, owned
 * by the caller; inputs and outputs must not alias.  Every compute call overwrites its whole
 * output, enqueues its kernels on `stream`, performs no allocation and no host
 * synchronisation, and returns a status (no exceptions cross this boundary).  A plan is
 * immutable after creation; calls on different streams may run concurrently when each has
 * its own workspace.
 */
#ifndef SYNO_H
#define SYNO_H

#include <stddef.h>
#include <stdint.h>
#include <hip/hip_runtime_api.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct syno_plan syno_plan;

typedef enum {
  SYNO_OK = 0,
  SYNO_ERR_NULL = 1,          /* a required pointer is NULL */
  SYNO_ERR_INVALID_DESC = 2,  /* the graph is not a valid pGraph (see syno_plan_create) */
  SYNO_ERR_SHAPE = 3,         /* an argument (index, count, selector) is out of range */
  SYNO_ERR_UNSUPPORTED = 4,   /* valid, but outside what the library lowers */
  SYNO_ERR_WORKSPACE = 5,     /* workspace required but NULL */
  SYNO_ERR_HIP = 6,           /* the HIP runtime reported an error at launch */
  SYNO_ERR_SCRATCH = 7        /* the call needs more scratch memory than the library's static buffer holds */
} syno_status;

typedef enum { SYNO_F32 = 0, SYNO_BF16 = 1 } syno_dtype;

/* Table 1 of the paper, bottom <- top.  i, j are the bottom coordinates (`in`), the results
 * are the top coordinates (`out`).
 *   SPLIT   [i,j]:[G,B]  <- [B*i+j]:[G*B]
 *   MERGE B [i]:[N]      <- [i/B, i%B]:[N/B,B]           (B must divide N)
 *   SHIFT   [i]:[N]      <- [(i+s) mod N]:[N]            (paper: s = 1; see `param`, `shift_by`)
 *   EXPAND  [i]:[C]      <- nothing                       (the output is repeated along i)
 *   UNFOLD  [i,j]:[N,K]  <- [i+j-K/2]:[N]                (floored K/2; out of range -> term dropped)
 *   STRIDE S[i]:[K]      <- [S*i]:[S*K]
 *   REDUCE N nothing     <- a new sum iterator of domain N
 *   SHARE   [i]:[N]      <- ([i],[i])                     (out[0] goes on towards X, out[1] to W)
 */
typedef enum {
  SYNO_SPLIT = 0, SYNO_MERGE = 1, SYNO_SHIFT = 2, SYNO_EXPAND = 3,
  SYNO_UNFOLD = 4, SYNO_STRIDE = 5, SYNO_REDUCE = 6, SYNO_SHARE = 7
} syno_prim_kind;

typedef struct {
  const char* name;   /* for messages only; may be NULL */
  int64_t size;       /* > 0 */
} syno_dim;

typedef struct {
  syno_prim_kind kind;
  int32_t in[2];        /* coordinate ids consumed (bottom side); unused slots are -1 */
  int32_t out[2];       /* coordinate ids produced (top side), each a fresh id; unused are -1 */
  int64_t param;        /* MERGE: B.  STRIDE: S.  REDUCE: N.  SHIFT: constant offset s (any sign) */
  int32_t shift_by;     /* SHIFT only: id of a coordinate whose value is read (not consumed), or -1 */
  int64_t shift_coef;   /* SHIFT only: the offset is s + shift_coef * value(shift_by) */
} syno_prim;

/* Optional overrides of the planner's choices, for verification and tuning (every field 0 = the planner
 * decides).  They select among code paths that compute the same operator; none changes a result beyond
 * the summation order.  Read once, while the plan is built.
 *   kernel_policy   1: every pass runs on the generic index-program kernels
 *   mfma_variant    1 + index of the contraction kernel's tile variant (forward and backward-data), or -1 for the
 *                   row-streaming member of the family (bf16, at most 64 channels per group);
 *                   mfma_rows = output rows per workgroup tile.  Ignored unless the pair fits the operator.
 *   mfma_taps       1: one window tap per inner step even where three would be taken
 *   mfma_splits     number of workgroups that share one output tile of the contraction kernel, each summing a
 *                   range of the reduced channels; their partial results go to the workspace and a second kernel
 *                   adds them in a fixed order (fp32 results only; by itself the planner splits only reductions
 *                   over thousands of channels whose tiles would not fill the GPU)
 *   dw_workgroups   target number of workgroups of the backward-weight contraction (split of the pixel axis)
 *   view_workgroups cap on the grid of the view kernel
 *   clock_probe     measurement aid (device memory, 4 x int64 per workgroup of the launch, owned by the caller, or
 *                   NULL): the first thread of every workgroup of the contraction kernel (forward and backward-data)
 *                   leaves the constant 100 MHz timestamp counter and the shader clock counter there on entry
 *                   ([0], [1]) and on exit ([2], [3]); the ratio of the two differences is the clock the kernel
 *                   ran at.  Results are not affected. */
typedef struct {
  int32_t kernel_policy;
  int32_t mfma_variant, mfma_rows, mfma_taps;
  int32_t dw_workgroups;
  int32_t view_workgroups;
  int32_t mfma_splits;
  void* clock_probe;
} syno_plan_options;

/* Coordinate ids 0..n_out-1 are the output iterators in the layout order of `out`; primitives
 * are applied in array order (bottom-up) and may only consume ids defined before them.  Every
 * coordinate must be consumed exactly once: by one primitive, or as one axis of X or of W. */
typedef struct {
  int32_t n_out;   const syno_dim*  out_dims;
  int32_t n_prim;  const syno_prim* prims;
  int32_t n_in;    const int32_t*   input_coords;    /* axes of X, outermost first */
  int32_t n_w;     const int32_t*   weight_coords;   /* axes of W, outermost first (may be 0: W is one element) */
  syno_dtype in_dtype;    /* element type of X, W and G */
  syno_dtype out_dtype;   /* element type of out and dX; accumulation is fp32; dW is always fp32 */
  const syno_plan_options* options;   /* NULL: defaults */
  /* Further weights W_1, W_2, ... (Fig. 7: Operator 1 multiplies two): out[o] = sum_r X[f]*W[g]*W_1[g_1]*...
   * more_weight_coords lists their axes one weight after the other, more_weight_ranks[i] axes each.  Such an
   * operator is evaluated in stages (syno_chain_create_materialized); syno_plan_create refuses it. */
  int32_t n_more_weights;  const int32_t* more_weight_ranks;  const int32_t* more_weight_coords;
} syno_desc;

/* Which of the three contractions a selector argument names. */
enum { SYNO_FWD = 0, SYNO_BWD_DATA = 1, SYNO_BWD_WEIGHT = 2 };

/* Build a plan (host only; copies everything it needs out of `desc`).
 * SYNO_ERR_INVALID_DESC: unknown / redefined / twice- or never-consumed coordinate, non-positive
 * size, Merge factor not dividing its domain, a Reduce iterator fed straight into Expand.
 * SYNO_ERR_UNSUPPORTED: a tensor with more than 2^31-1 elements, more than 8 axes or 24 distinct
 * coordinates, a pass that would sum more than 2^31-1 points per element, or a graph whose gradient index
 * maps the planner cannot invert (e.g. both copies of a Shared coordinate reaching X: a diagonal). */
syno_status syno_plan_create(const syno_desc* desc, syno_plan** plan);
syno_status syno_plan_destroy(syno_plan* plan);

/* out[o] = sum_r X[f(o,r)] * W[g(o,r)]   (section 5.3; Listing 1 for the convolution). */
syno_status syno_forward(const syno_plan* plan, const void* X, const void* W, void* out,
                         void* workspace, hipStream_t stream);
/* dX[x] = sum over valid (o,r) with f(o,r)=x of G[o]*W[g(o,r)]; elements no term reaches are
 * written as 0.  The adjoint of the forward map in X (section 5.2: the primitives are differentiable). */
syno_status syno_backward_data(const syno_plan* plan, const void* G, const void* W, void* dX,
                               void* workspace, hipStream_t stream);
/* dW[w] = sum over valid (o,r) with g(o,r)=w of G[o]*X[f(o,r)], fp32.  The adjoint in W. */
syno_status syno_backward_weight(const syno_plan* plan, const void* X, const void* G, void* dW,
                                 void* workspace, hipStream_t stream);

/* syno_backward_weight for callers that cannot allocate or pass device memory of their own (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the split partial sums live in a
 * buffer inside the library, SYNO_STATIC_SCRATCH_BYTES of static device memory per GPU, instead of a caller's
 * workspace.  Same result as syno_backward_weight, bit for bit.  Allocates nothing and never synchronises.
 * SYNO_ERR_SCRATCH when syno_plan_workspace_bytes(plan, SYNO_BWD_WEIGHT) exceeds the buffer.  All calls on one
 * GPU share the one buffer: calls that may overlap on a GPU (different streams or threads) race. */
#define SYNO_STATIC_SCRATCH_BYTES (32u << 20)
syno_status syno_backward_weight_static(const syno_plan* plan, const void* X, const void* G, void* dW,
                                        hipStream_t stream);

/* Bytes of device workspace call `which` needs (0: `workspace` may be NULL). */
syno_status syno_plan_workspace_bytes(const syno_plan* plan, int which, size_t* bytes);

/* Derived shapes.  Each array must have room for 8 entries; ranks are returned. */
syno_status syno_plan_shapes(const syno_plan* plan, int32_t* x_rank, int64_t* x_shape,
                             int32_t* w_rank, int64_t* w_shape, int32_t* out_rank, int64_t* out_shape);

/* Name of the kernel family call `which` dispatches to (static string, never NULL for a valid plan). */
const char* syno_plan_kernel(const syno_plan* plan, int which);

/* Human-readable summary of how call `which` will be launched (kernel family, tile shape, grid, LDS),
 * written NUL-terminated into buf[0..size).  For logs and tests; the format is not an interface. */
syno_status syno_plan_describe(const syno_plan* plan, int which, char* buf, size_t size);

/* Verification aid (not on the hot path): the index maps of the three contractions, evaluated on
 * the device from the same lowered tables the generic kernels use.
 * Each contraction `which` enumerates (target element t, free point q):
 *   FWD:        t = flat index into out, q = flat Reduce point (Reduce iterators in graph order,
 *               row-major)                      -> a_off = offset into X, b_off = offset into W
 *   BWD_DATA:   t = flat index into dX, q < free_size -> a_off = offset into G, b_off = offset into W
 *   BWD_WEIGHT: t = flat index into dW, q < free_size -> a_off = offset into G, b_off = offset into X
 * A point whose term does not exist yields -1 in both.  t_flat, q_flat, a_off, b_off are DEVICE
 * arrays of n entries. */
syno_status syno_plan_free_size(const syno_plan* plan, int which, int64_t* free_size);
syno_status syno_debug_gather(const syno_plan* plan, int which, const int64_t* t_flat, const int64_t* q_flat,
                              int64_t n, int32_t* a_off, int32_t* b_off, hipStream_t stream);

/* The same maps evaluated on the HOST from the same tables (all four arrays are host pointers); lets a
 * plan be checked on a machine without a GPU.  Index arithmetic only: no tensor data is touched. */
syno_status syno_debug_gather_host(const syno_plan* plan, int which, const int64_t* t_flat, const int64_t* q_flat,
                                   int64_t n, int32_t* a_off, int32_t* b_off);

/* Measurement aid (not on any operator's path): a kernel of `workgroups` x 4 waves that only issues 16x16 MFMAs of
 * the given input type, `iters` x 16 per wave, so that a benchmark can print the matrix-core rate the device
 * sustains beside the datasheet peak.  `out` is a DEVICE array of workgroups*256 floats (overwritten); *flop
 * receives the floating-point operations the launch performs. */
syno_status syno_debug_mfma_rate(syno_dtype dtype, int32_t iters, int32_t workgroups, float* out, int64_t* flop,
                                 hipStream_t stream);

/* ---- Operators evaluated in stages ---------------------------------------------------------------
 * The materialised-reduction pass of the paper's code-generation section cuts a pGraph with several
 * weights into sub-graphs whose results are stored, so that a Reduce above a one-to-many primitive is
 * evaluated once; Operator 1 (Fig. 7) becomes two such stages.  A chain is n_stages >= 1 single-weight
 * pGraphs: the data input of stage i+1 is the output of stage i (equal element count and element type;
 * the memory is reinterpreted row-major in stage i+1's input shape).
 *
 * W, act, dW are HOST arrays of DEVICE pointers: W[i] / dW[i] belong to stage i, act[i] (i < n_stages-1) is
 * the output of stage i.  The caller owns the act buffers: the forward call writes them and the backward
 * call reads them again (saved activations); with one stage `act` may be NULL. */
typedef struct syno_chain syno_chain;

/* Plans every stage.  Errors of syno_plan_create apply per stage; SYNO_ERR_SHAPE when consecutive stages do
 * not fit (element count or element type), or n_stages is outside 1..8. */
syno_status syno_chain_create(const syno_desc* stages, int32_t n_stages, syno_chain** chain);
/* The materialised-reduction pass itself (code-generation section; its Fig. shows Y[i] = sum_{ik,is} X[..] cut
 * into Z = sum_is, Y = sum_ik Z): for every Reduce of ONE single-weight pGraph the primitives between it and the
 * tensors form a candidate first stage whose result Z is stored; the cut with the fewest multiply-adds is taken
 * when it beats the single loop nest, and the rest of the graph is cut again.  The chain has 1..8 stages; every
 * stage has at most one weight (syno_chain_stage_weight; with a single-weight graph exactly one stage, also named by
 * syno_chain_weight_stage, keeps it): in the W and dW arrays of the forward and backward calls only the entries of
 * stages with a weight are read or written.  A graph with several weights must come apart into single-weight stages
 * this way (a first stage takes a weight together with the Shares that feed it, followed as the graph writes them),
 * else SYNO_ERR_UNSUPPORTED.  Graphs with a Shift that reads another coordinate are left whole.  Intermediates take
 * the graph's input element type. */
syno_status syno_chain_create_materialized(const syno_desc* desc, syno_chain** chain);
/* Stage that takes the caller's weight, or -1 when every stage has its own (syno_chain_create). */
int32_t syno_chain_weight_stage(const syno_chain* chain);
/* Which of the graph's weights (0 = W, 1.. = the further ones) stage `stage` multiplies with, or -1 when it has
 * none; chains from syno_chain_create: the stage's own index.  The W and dW arrays of the forward and backward calls
 * are indexed by STAGE: entry i belongs to the weight this function names for stage i. */
int32_t syno_chain_stage_weight(const syno_chain* chain, int32_t stage);
syno_status syno_chain_destroy(syno_chain* chain);
/* Number of stages, and the plan of one stage (borrowed; valid until the chain is destroyed; NULL when out of range). */
int32_t syno_chain_stages(const syno_chain* chain);
const syno_plan* syno_chain_plan(const syno_chain* chain, int32_t stage);
/* Device workspace of the forward sweep (which = 0) or the backward sweep (which = 1). */
syno_status syno_chain_workspace_bytes(const syno_chain* chain, int which, size_t* bytes);
/* out = stage[n-1](... stage[0](X, W[0]) ..., W[n-1]); the stages run in order on `stream`. */
syno_status syno_chain_forward(const syno_chain* chain, const void* X, const void* const* W, void* const* act,
                               void* out, void* workspace, hipStream_t stream);
/* Gradients of L = sum(out*G) by the chain rule, last stage first: dW[i] (fp32) for every stage and dX (may
 * be NULL: not computed).  G has the last stage's in_dtype.  Intermediate gradients live in the workspace, in the
 * input element type of the stage that consumes them (so a bf16 chain with an fp32 result runs its gradients in
 * bf16 between the stages).  dX has the first stage's out_dtype; for chains written by
 * syno_chain_create_materialized, the graph's out_dtype. */
syno_status syno_chain_backward(const syno_chain* chain, const void* X, const void* const* W,
                                const void* const* act, const void* G, void* dX, void* const* dW,
                                void* workspace, hipStream_t stream);

const char* syno_status_string(syno_status s);

#ifdef __cplusplus
}
#endif
#endif /* SYNO_H */
