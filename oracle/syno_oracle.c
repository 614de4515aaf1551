/*
 * CPU checker for synthesized operators.  TEST INFRASTRUCTURE ONLY: the tests, the
 * smoke check and the benchmark's CPU-baseline leg call it; the GPU library never does
 * and shares no code with it.
 *
 * What it computes is the plain definition.  An operator is a primitive graph
 * (section 5.1, Fig. 2): the output iterators are the bottom coordinates, every
 * primitive of Table 1 turns bottom coordinates into top coordinates, and the top
 * coordinates index the data input X and the weight W (section 5.3: the operator of a
 * pGraph is obtained by evaluating its coordinates from the bottom up with Table 1 and
 * indexing the tensors with the results).  Each Reduce adds
 * a sum loop, each Share multiplies the two tensors it indexes, so
 *
 *     out[o] = sum over all Reduce iterators r of  X[f(o,r)] * W[g(o,r)]
 *
 * in the loop-nest form of Listing 1.  Accumulation is in double precision.
 *
 * Readings where the paper is silent (each also listed in the design notes):
 *   - Unfold clips what falls outside the domain (Table 1 caption): here the term is
 *     dropped, i.e. zero padding, as the padded unfold of Listing 3 does.
 *   - K/2 in Unfold is the floored integer quotient.
 *   - Shift is generalised from (i+1)%N to (i + s + coef*value(by)) mod N with the
 *     non-negative remainder; s=1, no `by`, is the paper's primitive.
 *   - A term is valid iff every Unfold on its path is in range; the decision is taken at
 *     the Unfold and later primitives are only evaluated on valid terms.
 *   - Reduce is a pure sum (Table 2's AvgPool1d example has no 1/s).
 *   - Expand: the output does not depend on the expanded iterator (Table 1: the
 *     coordinate is discarded).
 *   - The backward pass is the adjoint of the bilinear map above (the paper only states
 *     that the primitives are differentiable, section 5.2): with L = sum_o out[o]*G[o],
 *     dX[f(o,r)] += G[o]*W[g(o,r)] and dW[g(o,r)] += G[o]*X[f(o,r)] over all valid (o,r).
 *
 * Descriptor wire format (int64 words), private to this file and its Python wrapper:
 *   n_out, size[n_out],
 *   n_prim, n_prim x {kind, in0, in1, out0, out1, param, shift_by, shift_coef},
 *   n_in, coord[n_in], n_w, coord[n_w] [, n_more, n_more x {n_wk, coord[n_wk]}]
 * The optional tail lists further weights: an operator may multiply several weights (Operator 1 of the paper,
 * Fig. 7, has two: each Share hands one copy of a coordinate to one of them).  Then
 *     out[o] = sum_r X[f(o,r)] * W_0[g_0(o,r)] * W_1[g_1(o,r)] * ...
 * kind: 0 Split 1 Merge 2 Shift 3 Expand 4 Unfold 5 Stride 6 Reduce 7 Share.
 * Coordinate ids 0..n_out-1 are the output iterators; unused slots are -1.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define MAXC 96
#define MAXP 64
#define MAXD 16
#define MAXW 4

enum { K_SPLIT = 0, K_MERGE, K_SHIFT, K_EXPAND, K_UNFOLD, K_STRIDE, K_REDUCE, K_SHARE };

enum {
  ORACLE_OK = 0,
  ORACLE_ERR_FORMAT = -1,     /* truncated or oversized descriptor */
  ORACLE_ERR_COORD = -2,      /* unknown id, id defined twice, consumed twice or never */
  ORACLE_ERR_DOMAIN = -3,     /* non-positive size, Merge factor not dividing the domain */
  ORACLE_ERR_FUTILE = -4      /* a Reduce iterator fed straight into Expand */
};

typedef struct {
  int kind, in0, in1, out0, out1, shift_by;
  int64_t param, shift_coef;
} prim_t;

typedef struct {
  int n_out;
  int64_t out_size[MAXD];
  int n_prim;
  prim_t prim[MAXP];
  int n_in, in_coord[MAXD];
  int n_w, w_coord[MAXD];
  int n_more;                          /* further weights (the first one is w_coord) */
  int m_n[MAXW], m_coord[MAXW][MAXD];
  int64_t m_elems[MAXW], m_stride[MAXW][MAXD];
  /* derived */
  int64_t dom[MAXC];
  int n_red;
  int64_t red_size[MAXP];
  int64_t n_o, n_r, x_elems, w_elems;
  int64_t x_stride[MAXD], w_stride[MAXD];
} op_t;

static int parse(const int64_t *d, int64_t len, op_t *op) {
  int64_t p = 0;
  int defined[MAXC], used[MAXC], from_reduce[MAXC];
  memset(op, 0, sizeof(*op));
  memset(defined, 0, sizeof(defined));
  memset(used, 0, sizeof(used));
  memset(from_reduce, 0, sizeof(from_reduce));
#define NEED(k) do { if (p + (k) > len) return ORACLE_ERR_FORMAT; } while (0)
  NEED(1);
  op->n_out = (int)d[p++];
  if (op->n_out < 0 || op->n_out > MAXD) return ORACLE_ERR_FORMAT;
  NEED(op->n_out);
  op->n_o = 1;
  for (int i = 0; i < op->n_out; ++i) {
    op->out_size[i] = d[p++];
    if (op->out_size[i] <= 0) return ORACLE_ERR_DOMAIN;
    op->dom[i] = op->out_size[i];
    defined[i] = 1;
    op->n_o *= op->out_size[i];
  }
  NEED(1);
  op->n_prim = (int)d[p++];
  if (op->n_prim < 0 || op->n_prim > MAXP) return ORACLE_ERR_FORMAT;
  op->n_r = 1;
  for (int k = 0; k < op->n_prim; ++k) {
    prim_t *q = &op->prim[k];
    NEED(8);
    q->kind = (int)d[p++];
    q->in0 = (int)d[p++];
    q->in1 = (int)d[p++];
    q->out0 = (int)d[p++];
    q->out1 = (int)d[p++];
    q->param = d[p++];
    q->shift_by = (int)d[p++];
    q->shift_coef = d[p++];
    int nin, nout;
    switch (q->kind) {
      case K_SPLIT:  nin = 2; nout = 1; break;
      case K_MERGE:  nin = 1; nout = 2; break;
      case K_SHIFT:  nin = 1; nout = 1; break;
      case K_EXPAND: nin = 1; nout = 0; break;
      case K_UNFOLD: nin = 2; nout = 1; break;
      case K_STRIDE: nin = 1; nout = 1; break;
      case K_REDUCE: nin = 0; nout = 1; break;
      case K_SHARE:  nin = 1; nout = 2; break;
      default: return ORACLE_ERR_FORMAT;
    }
    int ins[2] = { q->in0, q->in1 }, outs[2] = { q->out0, q->out1 };
    for (int t = 0; t < 2; ++t) {
      if (t < nin) {
        if (ins[t] < 0 || ins[t] >= MAXC || !defined[ins[t]] || used[ins[t]]) return ORACLE_ERR_COORD;
        used[ins[t]] = 1;
      } else if (ins[t] != -1) return ORACLE_ERR_COORD;
      if (t < nout) {
        if (outs[t] < 0 || outs[t] >= MAXC || defined[outs[t]]) return ORACLE_ERR_COORD;
        defined[outs[t]] = 1;
      } else if (outs[t] != -1) return ORACLE_ERR_COORD;
    }
    switch (q->kind) {
      case K_SPLIT:  op->dom[q->out0] = op->dom[q->in0] * op->dom[q->in1]; break;
      case K_MERGE:
        if (q->param <= 0 || op->dom[q->in0] % q->param != 0) return ORACLE_ERR_DOMAIN;
        op->dom[q->out0] = op->dom[q->in0] / q->param;
        op->dom[q->out1] = q->param;
        break;
      case K_SHIFT:
        if (q->shift_by != -1 && (q->shift_by < 0 || q->shift_by >= MAXC || !defined[q->shift_by]))
          return ORACLE_ERR_COORD;
        op->dom[q->out0] = op->dom[q->in0];
        break;
      case K_EXPAND:
        if (from_reduce[q->in0]) return ORACLE_ERR_FUTILE;
        break;
      case K_UNFOLD: op->dom[q->out0] = op->dom[q->in0]; break;
      case K_STRIDE:
        if (q->param <= 0) return ORACLE_ERR_DOMAIN;
        op->dom[q->out0] = q->param * op->dom[q->in0];
        break;
      case K_REDUCE:
        if (q->param <= 0) return ORACLE_ERR_DOMAIN;
        op->dom[q->out0] = q->param;
        from_reduce[q->out0] = 1;
        op->red_size[op->n_red++] = q->param;
        op->n_r *= q->param;
        break;
      case K_SHARE:
        op->dom[q->out0] = op->dom[q->in0];
        op->dom[q->out1] = op->dom[q->in0];
        break;
    }
  }
  NEED(1);
  op->n_in = (int)d[p++];
  if (op->n_in < 0 || op->n_in > MAXD) return ORACLE_ERR_FORMAT;
  NEED(op->n_in);
  for (int i = 0; i < op->n_in; ++i) {
    int c = (int)d[p++];
    if (c < 0 || c >= MAXC || !defined[c] || used[c]) return ORACLE_ERR_COORD;
    used[c] = 1;
    op->in_coord[i] = c;
  }
  NEED(1);
  op->n_w = (int)d[p++];
  if (op->n_w < 0 || op->n_w > MAXD) return ORACLE_ERR_FORMAT;
  NEED(op->n_w);
  for (int i = 0; i < op->n_w; ++i) {
    int c = (int)d[p++];
    if (c < 0 || c >= MAXC || !defined[c] || used[c]) return ORACLE_ERR_COORD;
    used[c] = 1;
    op->w_coord[i] = c;
  }
  if (p != len) {                       /* further weights */
    NEED(1);
    op->n_more = (int)d[p++];
    if (op->n_more < 1 || op->n_more > MAXW) return ORACLE_ERR_FORMAT;
    for (int k = 0; k < op->n_more; ++k) {
      NEED(1);
      op->m_n[k] = (int)d[p++];
      if (op->m_n[k] < 0 || op->m_n[k] > MAXD) return ORACLE_ERR_FORMAT;
      NEED(op->m_n[k]);
      for (int i = 0; i < op->m_n[k]; ++i) {
        int c = (int)d[p++];
        if (c < 0 || c >= MAXC || !defined[c] || used[c]) return ORACLE_ERR_COORD;
        used[c] = 1;
        op->m_coord[k][i] = c;
      }
    }
    if (p != len) return ORACLE_ERR_FORMAT;
  }
  for (int c = 0; c < MAXC; ++c)
    if (defined[c] && !used[c]) return ORACLE_ERR_COORD;   /* a coordinate nobody consumes */
  /* row-major strides of X and W */
  op->x_elems = 1;
  for (int i = op->n_in - 1; i >= 0; --i) {
    op->x_stride[i] = op->x_elems;
    op->x_elems *= op->dom[op->in_coord[i]];
  }
  op->w_elems = 1;
  for (int i = op->n_w - 1; i >= 0; --i) {
    op->w_stride[i] = op->w_elems;
    op->w_elems *= op->dom[op->w_coord[i]];
  }
  for (int k = 0; k < op->n_more; ++k) {
    op->m_elems[k] = 1;
    for (int i = op->m_n[k] - 1; i >= 0; --i) {
      op->m_stride[k][i] = op->m_elems[k];
      op->m_elems[k] *= op->dom[op->m_coord[k][i]];
    }
  }
  return ORACLE_OK;
#undef NEED
}

static int64_t pos_mod(int64_t a, int64_t n) {
  int64_t m = a % n;
  return m < 0 ? m + n : m;
}

/* Evaluate every coordinate for one point (o, r) of the loop nest, bottom-up (Table 1).
 * Returns 1 and the flat offsets into X and W if the term exists; 0 and both offsets -1 if
 * an Unfold on the path is out of range. */
static int eval_point_all(const op_t *op, const int64_t *o, const int64_t *r, int64_t *x_off, int64_t *w_off,
                          int64_t *m_off) {
  int64_t val[MAXC];
  int valid = 1, nr = 0;
  for (int i = 0; i < op->n_out; ++i) val[i] = o[i];
  for (int k = 0; k < op->n_prim; ++k) {
    const prim_t *q = &op->prim[k];
    switch (q->kind) {
      case K_SPLIT:                       /* [i, j]: [G, B]  <-  [B*i + j]: [G*B] */
        val[q->out0] = op->dom[q->in1] * val[q->in0] + val[q->in1];
        break;
      case K_MERGE:                       /* [i]: [N]  <-  [i / B, i % B]: [N/B, B] */
        val[q->out0] = valid ? val[q->in0] / q->param : 0;
        val[q->out1] = valid ? val[q->in0] % q->param : 0;
        break;
      case K_SHIFT: {                     /* [i]: [N]  <-  [(i + s) % N]: [N] */
        int64_t s = q->param;
        if (q->shift_by >= 0) s += q->shift_coef * val[q->shift_by];
        val[q->out0] = valid ? pos_mod(val[q->in0] + s, op->dom[q->in0]) : 0;
        break;
      }
      case K_EXPAND:                      /* [i]: [C]  <-  []: [] */
        break;
      case K_UNFOLD: {                    /* [i, j]: [N, K]  <-  [i + j - K/2]: [N], clipped */
        int64_t K = op->dom[q->in1], N = op->dom[q->in0];
        int64_t v = val[q->in0] + val[q->in1] - K / 2;
        if (v < 0 || v >= N) { valid = 0; v = 0; }
        val[q->out0] = v;
        break;
      }
      case K_STRIDE:                      /* [i]: [K]  <-  [S*i]: [S*K] */
        val[q->out0] = q->param * val[q->in0];
        break;
      case K_REDUCE:                      /* []: []  <-  sum_i [i]: [N] */
        val[q->out0] = r[nr++];
        break;
      case K_SHARE:                       /* [i]: [N]  <-  ([i], [i]) */
        val[q->out0] = val[q->in0];
        val[q->out1] = val[q->in0];
        break;
    }
  }
  int64_t xo = 0, wo = 0;
  for (int i = 0; i < op->n_in; ++i) xo += val[op->in_coord[i]] * op->x_stride[i];
  for (int i = 0; i < op->n_w; ++i) wo += val[op->w_coord[i]] * op->w_stride[i];
  *x_off = valid ? xo : -1;
  *w_off = valid ? wo : -1;
  if (m_off)
    for (int k = 0; k < op->n_more; ++k) {
      int64_t mo = 0;
      for (int i = 0; i < op->m_n[k]; ++i) mo += val[op->m_coord[k][i]] * op->m_stride[k][i];
      m_off[k] = valid ? mo : -1;
    }
  return valid;
}

static int eval_point(const op_t *op, const int64_t *o, const int64_t *r, int64_t *x_off, int64_t *w_off) {
  return eval_point_all(op, o, r, x_off, w_off, NULL);
}

static void unflatten(int64_t flat, int n, const int64_t *size, int64_t *idx) {
  for (int i = n - 1; i >= 0; --i) {
    idx[i] = flat % size[i];
    flat /= size[i];
  }
}

/* ---------------------------------------------------------------------------------- */
/* Exported entry points.  All tensors are host arrays of doubles, row-major.          */
/* ---------------------------------------------------------------------------------- */

/* Validate and report the derived shapes.  x_shape / w_shape / red_shape have room for 16. */
int oracle_describe(const int64_t *desc, int64_t len, int64_t *x_rank, int64_t *x_shape, int64_t *w_rank,
                    int64_t *w_shape, int64_t *n_red, int64_t *red_shape) {
  op_t op;
  int rc = parse(desc, len, &op);
  if (rc) return rc;
  *x_rank = op.n_in;
  for (int i = 0; i < op.n_in; ++i) x_shape[i] = op.dom[op.in_coord[i]];
  *w_rank = op.n_w;
  for (int i = 0; i < op.n_w; ++i) w_shape[i] = op.dom[op.w_coord[i]];
  *n_red = op.n_red;
  for (int i = 0; i < op.n_red; ++i) red_shape[i] = op.red_size[i];
  return ORACLE_OK;
}

/* out[o] for every output point. */
int oracle_forward(const int64_t *desc, int64_t len, const double *X, const double *W, double *out) {
  op_t op;
  int rc = parse(desc, len, &op);
  if (rc) return rc;
  if (op.n_more) return ORACLE_ERR_FORMAT;     /* several weights: the _multi entry points */
#pragma omp parallel for schedule(static)
  for (int64_t of = 0; of < op.n_o; ++of) {
    int64_t o[MAXD], r[MAXP], xo, wo;
    unflatten(of, op.n_out, op.out_size, o);
    double acc = 0.0;
    for (int64_t rf = 0; rf < op.n_r; ++rf) {
      unflatten(rf, op.n_red, op.red_size, r);
      if (eval_point(&op, o, r, &xo, &wo)) acc += X[xo] * W[wo];
    }
    out[of] = acc;
  }
  return ORACLE_OK;
}

/* out[o] for the n listed flat output indices only. */
int oracle_forward_at(const int64_t *desc, int64_t len, const double *X, const double *W,
                      const int64_t *o_flat, int64_t n, double *out) {
  op_t op;
  int rc = parse(desc, len, &op);
  if (rc) return rc;
  if (op.n_more) return ORACLE_ERR_FORMAT;     /* several weights: the _multi entry points */
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < n; ++s) {
    int64_t o[MAXD], r[MAXP], xo, wo;
    unflatten(o_flat[s], op.n_out, op.out_size, o);
    double acc = 0.0;
    for (int64_t rf = 0; rf < op.n_r; ++rf) {
      unflatten(rf, op.n_red, op.red_size, r);
      if (eval_point(&op, o, r, &xo, &wo)) acc += X[xo] * W[wo];
    }
    out[s] = acc;
  }
  return ORACLE_OK;
}

/* dX and dW (either may be NULL) in scatter form over the same loop nest.
 * x_pick / w_pick, when not NULL, are maps flat index -> slot or -1: then only the picked
 * elements are accumulated, into dX[slot] / dW[slot] (used to check sampled elements of
 * problems too large to hold or finish in full). */
int oracle_backward(const int64_t *desc, int64_t len, const double *X, const double *W, const double *G,
                    double *dX, double *dW, const int64_t *x_pick, int64_t n_x_pick,
                    const int64_t *w_pick, int64_t n_w_pick) {
  op_t op;
  int rc = parse(desc, len, &op);
  if (rc) return rc;
  if (op.n_more) return ORACLE_ERR_FORMAT;     /* several weights: the _multi entry points */
  if (dX) memset(dX, 0, sizeof(double) * (size_t)(x_pick ? n_x_pick : op.x_elems));
  if (dW) memset(dW, 0, sizeof(double) * (size_t)(w_pick ? n_w_pick : op.w_elems));
#pragma omp parallel for schedule(static)
  for (int64_t of = 0; of < op.n_o; ++of) {
    int64_t o[MAXD], r[MAXP], xo, wo;
    unflatten(of, op.n_out, op.out_size, o);
    const double g = G[of];
    for (int64_t rf = 0; rf < op.n_r; ++rf) {
      unflatten(rf, op.n_red, op.red_size, r);
      if (!eval_point(&op, o, r, &xo, &wo)) continue;
      if (dX) {
        int64_t slot = x_pick ? x_pick[xo] : xo;
        if (slot >= 0) {
          double t = g * W[wo];
#pragma omp atomic
          dX[slot] += t;
        }
      }
      if (dW) {
        int64_t slot = w_pick ? w_pick[wo] : wo;
        if (slot >= 0) {
          double t = g * X[xo];
#pragma omp atomic
          dW[slot] += t;
        }
      }
    }
  }
  return ORACLE_OK;
}

/* Index map of the loop nest: for each listed point (o_flat, r_flat) the flat offsets into
 * X and W, or -1 for both when an Unfold is out of range. */
int oracle_gather_map(const int64_t *desc, int64_t len, const int64_t *o_flat, const int64_t *r_flat,
                      int64_t n, int32_t *x_off, int32_t *w_off) {
  op_t op;
  int rc = parse(desc, len, &op);
  if (rc) return rc;
  if (op.n_more) return ORACLE_ERR_FORMAT;     /* several weights: the _multi entry points */
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < n; ++s) {
    int64_t o[MAXD], r[MAXP], xo, wo;
    unflatten(o_flat[s], op.n_out, op.out_size, o);
    unflatten(r_flat[s], op.n_red, op.red_size, r);
    eval_point(&op, o, r, &xo, &wo);
    x_off[s] = (int32_t)xo;
    w_off[s] = (int32_t)wo;
  }
  return ORACLE_OK;
}

/* ---- operators with several weights: W[0] is the first weight, W[1..] the further ones ------------------------ */

/* Ranks and shapes of the further weights: shapes has room for MAXW x 16. */
int oracle_describe_more(const int64_t *desc, int64_t len, int64_t *n_more, int64_t *ranks, int64_t *shapes) {
  op_t op;
  int rc = parse(desc, len, &op);
  if (rc) return rc;
  *n_more = op.n_more;
  for (int k = 0; k < op.n_more; ++k) {
    ranks[k] = op.m_n[k];
    for (int i = 0; i < op.m_n[k]; ++i) shapes[16 * k + i] = op.dom[op.m_coord[k][i]];
  }
  return ORACLE_OK;
}

/* out[o] = sum_r X[f] * prod_k W_k[g_k]. */
int oracle_forward_multi(const int64_t *desc, int64_t len, const double *X, const double *const *W, double *out) {
  op_t op;
  int rc = parse(desc, len, &op);
  if (rc) return rc;
#pragma omp parallel for schedule(static)
  for (int64_t of = 0; of < op.n_o; ++of) {
    int64_t o[MAXD], r[MAXP], xo, wo, mo[MAXW];
    unflatten(of, op.n_out, op.out_size, o);
    double acc = 0.0;
    for (int64_t rf = 0; rf < op.n_r; ++rf) {
      unflatten(rf, op.n_red, op.red_size, r);
      if (!eval_point_all(&op, o, r, &xo, &wo, mo)) continue;
      double t = X[xo] * W[0][wo];
      for (int k = 0; k < op.n_more; ++k) t *= W[k + 1][mo[k]];
      acc += t;
    }
    out[of] = acc;
  }
  return ORACLE_OK;
}

/* Scatter-form gradients of L = sum_o out[o]*G[o]: every valid term adds G[o] times the product of the other
 * factors to dX and to each dW_k (any of which may be NULL). */
int oracle_backward_multi(const int64_t *desc, int64_t len, const double *X, const double *const *W, const double *G,
                          double *dX, double *const *dW) {
  op_t op;
  int rc = parse(desc, len, &op);
  if (rc) return rc;
  if (dX) memset(dX, 0, sizeof(double) * (size_t)op.x_elems);
  if (dW && dW[0]) memset(dW[0], 0, sizeof(double) * (size_t)op.w_elems);
  for (int k = 0; k < op.n_more; ++k)
    if (dW && dW[k + 1]) memset(dW[k + 1], 0, sizeof(double) * (size_t)op.m_elems[k]);
#pragma omp parallel for schedule(static)
  for (int64_t of = 0; of < op.n_o; ++of) {
    int64_t o[MAXD], r[MAXP], xo, wo, mo[MAXW];
    unflatten(of, op.n_out, op.out_size, o);
    const double g = G[of];
    for (int64_t rf = 0; rf < op.n_r; ++rf) {
      unflatten(rf, op.n_red, op.red_size, r);
      if (!eval_point_all(&op, o, r, &xo, &wo, mo)) continue;
      double f[MAXW + 2];                 /* the factors: X, W_0, W_1, ... */
      int nf = 2 + op.n_more;
      f[0] = X[xo]; f[1] = W[0][wo];
      for (int k = 0; k < op.n_more; ++k) f[2 + k] = W[k + 1][mo[k]];
      for (int i = 0; i < nf; ++i) {
        double *dst = i == 0 ? dX : (dW ? dW[i - 1] : NULL);
        if (!dst) continue;
        double t = g;
        for (int j = 0; j < nf; ++j) if (j != i) t *= f[j];
        int64_t slot = i == 0 ? xo : (i == 1 ? wo : mo[i - 2]);
#pragma omp atomic
        dst[slot] += t;
      }
    }
  }
  return ORACLE_OK;
}

/* Number of worker threads the loops above use (1 when built without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int oracle_threads(void) { return omp_get_max_threads(); }
#else
int oracle_threads(void) { return 1; }
#endif
