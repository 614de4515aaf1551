// Host planner: pGraph -> validated graph -> lowered index programs for the forward pass and the
// two gradients -> convolution-like form when the index map is affine -> kernel choice.
//
// Semantics follow Table 1 of the paper evaluated bottom-up (section 5.3).  The gradients are
// lowered as gathers: starting from the axes of the tensor being produced, every primitive is
// inverted where it is a bijection (Split, Merge, Shift), Unfold v = i + j - K/2 is solved for i
// once j is enumerated (with a range test), Stride v = S*i is solved when S divides v, and
// coordinates nothing determines are enumerated.
#include <algorithm>
#include <array>
#include <cstdlib>
#include <cstring>
#include <map>
#include <string>
#include <vector>

#include "plan.h"

namespace syno {
namespace {

constexpr int kMaxCoordId = 256;
constexpr int64_t kMaxElems = 2147483647LL;

struct Graph {
  int n_out = 0;
  std::vector<int64_t> dom;        // by coordinate id (0 where undefined)
  std::vector<int> slot;           // by coordinate id: value slot (Share copies share one)
  std::vector<syno_prim> prims;
  std::vector<int> in_coords, w_coords;
  std::vector<std::vector<int>> more_w;   // further weights
  int n_slots = 0;
  std::vector<int64_t> slot_dom;
  std::vector<int> reduce_coords;  // in graph order
  std::vector<int64_t> out_stride; // by output axis
  int64_t D(int c) const { return dom[c]; }
  int S(int c) const { return slot[c]; }
};

int arity_in(int kind) {
  switch (kind) {
    case SYNO_SPLIT: case SYNO_UNFOLD: return 2;
    case SYNO_REDUCE: return 0;
    default: return 1;
  }
}
int arity_out(int kind) {
  switch (kind) {
    case SYNO_MERGE: case SYNO_SHARE: return 2;
    case SYNO_EXPAND: return 0;
    default: return 1;
  }
}

syno_status parse_graph(const syno_desc* d, Graph& g, std::string* why) {
  auto bad = [&](const char* m) { if (why) *why = m; return SYNO_ERR_INVALID_DESC; };
  if (d->n_out < 0 || d->n_prim < 0 || d->n_in < 0 || d->n_w < 0) return bad("negative count");
  if ((d->n_out && !d->out_dims) || (d->n_prim && !d->prims) || (d->n_in && !d->input_coords) ||
      (d->n_w && !d->weight_coords))
    return SYNO_ERR_NULL;
  if (d->n_out > kMaxAxes || d->n_in > kMaxAxes || d->n_w > kMaxAxes) {
    if (why) *why = "more than 8 axes";
    return SYNO_ERR_UNSUPPORTED;
  }
  if (d->in_dtype != SYNO_F32 && d->in_dtype != SYNO_BF16) return bad("in_dtype");
  if (d->out_dtype != SYNO_F32 && d->out_dtype != SYNO_BF16) return bad("out_dtype");
  g.n_out = d->n_out;
  g.dom.assign(kMaxCoordId, 0);
  std::vector<char> defined(kMaxCoordId, 0), used(kMaxCoordId, 0), from_reduce(kMaxCoordId, 0);
  std::vector<int> parent(kMaxCoordId);
  for (int i = 0; i < kMaxCoordId; ++i) parent[i] = i;
  auto find = [&](int x) { while (parent[x] != x) x = parent[x] = parent[parent[x]]; return x; };
  for (int i = 0; i < d->n_out; ++i) {
    if (d->out_dims[i].size <= 0) return bad("output size <= 0");
    g.dom[i] = d->out_dims[i].size;
    defined[i] = 1;
  }
  for (int k = 0; k < d->n_prim; ++k) {
    const syno_prim& p = d->prims[k];
    if ((int)p.kind < 0 || (int)p.kind > SYNO_SHARE) return bad("unknown primitive");
    const int ni = arity_in(p.kind), no = arity_out(p.kind);
    for (int t = 0; t < 2; ++t) {
      if (t < ni) {
        const int c = p.in[t];
        if (c < 0 || c >= kMaxCoordId || !defined[c]) return bad("primitive consumes an undefined coordinate");
        if (used[c]) return bad("coordinate consumed twice");
        used[c] = 1;
      } else if (p.in[t] != -1) return bad("unused in slot must be -1");
      if (t < no) {
        const int c = p.out[t];
        if (c < 0 || c >= kMaxCoordId) return bad("coordinate id out of range");
        if (defined[c]) return bad("coordinate defined twice");
        defined[c] = 1;
      } else if (p.out[t] != -1) return bad("unused out slot must be -1");
    }
    switch (p.kind) {
      case SYNO_SPLIT: g.dom[p.out[0]] = g.dom[p.in[0]] * g.dom[p.in[1]]; break;
      case SYNO_MERGE:
        if (p.param <= 0 || g.dom[p.in[0]] % p.param) return bad("Merge factor must divide the domain");
        g.dom[p.out[0]] = g.dom[p.in[0]] / p.param;
        g.dom[p.out[1]] = p.param;
        break;
      case SYNO_SHIFT:
        if (p.shift_by != -1 && (p.shift_by < 0 || p.shift_by >= kMaxCoordId || !defined[p.shift_by]))
          return bad("shift_by names an undefined coordinate");
        g.dom[p.out[0]] = g.dom[p.in[0]];
        break;
      case SYNO_EXPAND:
        if (from_reduce[p.in[0]]) return bad("a Reduce iterator is fed straight into Expand");
        break;
      case SYNO_UNFOLD: g.dom[p.out[0]] = g.dom[p.in[0]]; break;
      case SYNO_STRIDE:
        if (p.param <= 0) return bad("Stride factor <= 0");
        g.dom[p.out[0]] = g.dom[p.in[0]] * p.param;
        break;
      case SYNO_REDUCE:
        if (p.param <= 0) return bad("Reduce size <= 0");
        g.dom[p.out[0]] = p.param;
        from_reduce[p.out[0]] = 1;
        g.reduce_coords.push_back(p.out[0]);
        break;
      case SYNO_SHARE:
        g.dom[p.out[0]] = g.dom[p.out[1]] = g.dom[p.in[0]];
        parent[find(p.out[0])] = find(p.in[0]);
        parent[find(p.out[1])] = find(p.in[0]);
        break;
    }
    for (int t = 0; t < no; ++t)
      if (g.dom[p.out[t]] > kMaxElems) { if (why) *why = "domain too large"; return SYNO_ERR_UNSUPPORTED; }
    g.prims.push_back(p);
  }
  for (int i = 0; i < d->n_in; ++i) {
    const int c = d->input_coords[i];
    if (c < 0 || c >= kMaxCoordId || !defined[c]) return bad("X axis names an undefined coordinate");
    if (used[c]) return bad("coordinate consumed twice");
    used[c] = 1;
    g.in_coords.push_back(c);
  }
  for (int i = 0; i < d->n_w; ++i) {
    const int c = d->weight_coords[i];
    if (c < 0 || c >= kMaxCoordId || !defined[c]) return bad("W axis names an undefined coordinate");
    if (used[c]) return bad("coordinate consumed twice");
    used[c] = 1;
    g.w_coords.push_back(c);
  }
  if (d->n_more_weights < 0 || d->n_more_weights > 3) return bad("count of further weights");
  if (d->n_more_weights && (!d->more_weight_ranks || !d->more_weight_coords)) return SYNO_ERR_NULL;
  for (int k = 0, at = 0; k < d->n_more_weights; ++k) {
    const int rank = d->more_weight_ranks[k];
    if (rank < 0 || rank > kMaxAxes) return bad("rank of a further weight");
    g.more_w.emplace_back();
    for (int i = 0; i < rank; ++i) {
      const int c = d->more_weight_coords[at++];
      if (c < 0 || c >= kMaxCoordId || !defined[c]) return bad("W axis names an undefined coordinate");
      if (used[c]) return bad("coordinate consumed twice");
      used[c] = 1;
      g.more_w.back().push_back(c);
    }
  }
  for (int c = 0; c < kMaxCoordId; ++c)
    if (defined[c] && !used[c]) return bad("coordinate never consumed");
  // slots
  g.slot.assign(kMaxCoordId, -1);
  std::map<int, int> root_slot;
  for (int c = 0; c < kMaxCoordId; ++c) {
    if (!defined[c]) continue;
    const int r = find(c);
    auto it = root_slot.find(r);
    if (it == root_slot.end()) {
      it = root_slot.emplace(r, g.n_slots++).first;
      g.slot_dom.push_back(g.dom[c]);
    }
    g.slot[c] = it->second;
  }
  if (g.n_slots > kMaxSlots || (int)g.prims.size() > kMaxOps) {
    if (why) *why = "graph too large";
    return SYNO_ERR_UNSUPPORTED;
  }
  g.out_stride.assign(g.n_out, 1);
  for (int i = g.n_out - 2; i >= 0; --i) g.out_stride[i] = g.out_stride[i + 1] * g.dom[i + 1];
  return SYNO_OK;
}

int32_t pos_mod(int64_t a, int64_t n) {
  int64_t m = a % n;
  return (int32_t)(m < 0 ? m + n : m);
}

// ---------------------------------------------------------------------------------------------
// Index-program construction
// ---------------------------------------------------------------------------------------------
struct Builder {
  const Graph& g;
  std::vector<char> known;        // by slot
  std::vector<IndexOp> ops;
  std::vector<int> free_slots;    // in the order they were chosen
  bool failed = false;
  explicit Builder(const Graph& gg) : g(gg), known(gg.n_slots, 0) {}
  bool K(int c) const { return known[g.S(c)]; }
  void set(int c) { known[g.S(c)] = 1; }
  void emit(int kind, int a, int b, int d0, int d1, int64_t p0, int64_t p1, int64_t p2) {
    IndexOp o{kind, a, b, d0, d1, (int32_t)p0, (int32_t)p1, (int32_t)p2};
    ops.push_back(o);
  }
};

// Try to process primitive k with what is known.  Returns true when it is finished.
bool step_prim(Builder& b, const syno_prim& p, bool* progress) {
  const Graph& g = b.g;
  auto S = [&](int c) { return g.S(c); };
  switch (p.kind) {
    case SYNO_SHARE: return true;                       // copies alias one slot
    case SYNO_REDUCE: return b.K(p.out[0]);
    case SYNO_EXPAND: return b.K(p.in[0]);
    case SYNO_SPLIT: {
      const int i = p.in[0], j = p.in[1], v = p.out[0];
      if (b.K(i) && b.K(j) && !b.K(v)) {
        b.emit(OP_MULADD, S(i), S(j), S(v), -1, g.D(j), 0, 0);
        b.set(v);
      } else if (b.K(v) && !b.K(i) && !b.K(j)) {
        if (S(i) == S(j)) { b.failed = true; return false; }   // two copies of one Shared coordinate: determined twice
        b.emit(OP_DIVMOD, S(v), -1, S(i), S(j), g.D(j), (int32_t)division_magic(g.D(j)), 0);
        b.set(i); b.set(j);
      } else {
        if (b.K(v) && (b.K(i) || b.K(j))) b.failed = true;   // determined twice
        return false;
      }
      *progress = true;
      return true;
    }
    case SYNO_MERGE: {
      const int i = p.in[0], q = p.out[0], r = p.out[1];
      if (b.K(i) && !b.K(q) && !b.K(r)) {
        b.emit(OP_DIVMOD, S(i), -1, S(q), S(r), p.param, (int32_t)division_magic(p.param), 0);
        b.set(q); b.set(r);
      } else if (b.K(q) && b.K(r) && !b.K(i)) {
        b.emit(OP_MULADD, S(q), S(r), S(i), -1, p.param, 0, 0);
        b.set(i);
      } else {
        if (b.K(i) && (b.K(q) || b.K(r))) b.failed = true;
        return false;
      }
      *progress = true;
      return true;
    }
    case SYNO_SHIFT: {
      const int i = p.in[0], v = p.out[0], by = p.shift_by;
      if (by >= 0 && !b.K(by)) return false;
      const int64_t N = g.D(i);
      const int bs = by >= 0 ? S(by) : -1;
      const int64_t coef = by >= 0 ? p.shift_coef : 0;
      if (b.K(i) && !b.K(v)) {
        b.emit(OP_SHIFT, S(i), bs >= 0 ? bs : S(i), S(v), -1, N, pos_mod(p.param, N), pos_mod(coef, N));
        b.set(v);
      } else if (b.K(v) && !b.K(i)) {
        b.emit(OP_SHIFT, S(v), bs >= 0 ? bs : S(v), S(i), -1, N, pos_mod(-p.param, N), pos_mod(-coef, N));
        b.set(i);
      } else {
        if (b.K(i) && b.K(v)) b.failed = true;
        return false;
      }
      *progress = true;
      return true;
    }
    case SYNO_UNFOLD: {
      const int i = p.in[0], j = p.in[1], v = p.out[0];
      const int64_t N = g.D(i), Kd = g.D(j);
      if (b.K(i) && b.K(j) && !b.K(v)) {
        b.emit(OP_ADDCHK, S(i), S(j), S(v), -1, N, -(Kd / 2), 1);
        b.set(v);
      } else if (b.K(v) && b.K(j) && !b.K(i)) {
        b.emit(OP_ADDCHK, S(v), S(j), S(i), -1, N, Kd / 2, -1);      // i = v - j + K/2 within [0,N)
        b.set(i);
      } else if (b.K(v) && b.K(i) && !b.K(j)) {
        b.emit(OP_ADDCHK, S(v), S(i), S(j), -1, Kd, Kd / 2, -1);     // j = v - i + K/2 within [0,K)
        b.set(j);
      } else {
        if (b.K(v) && b.K(i) && b.K(j)) b.failed = true;
        return false;
      }
      *progress = true;
      return true;
    }
    case SYNO_STRIDE: {
      const int i = p.in[0], v = p.out[0];
      if (b.K(i) && !b.K(v)) {
        b.emit(OP_MUL, S(i), -1, S(v), -1, p.param, 0, 0);
        b.set(v);
      } else if (b.K(v) && !b.K(i)) {
        b.emit(OP_DIVCHK, S(v), -1, S(i), -1, p.param, (int32_t)division_magic(p.param), 0);
        b.set(i);
      } else {
        if (b.K(i) && b.K(v)) b.failed = true;
        return false;
      }
      *progress = true;
      return true;
    }
  }
  return false;
}

// Coordinate to enumerate when nothing more can be derived: prefer one that unblocks a
// half-determined primitive (smallest domain first), else any undetermined iterator.
int pick_free(const Builder& b, const std::vector<char>& done) {
  const Graph& g = b.g;
  int best = -1;
  auto consider = [&](int c) {
    if (c >= 0 && !b.K(c) && (best < 0 || g.D(c) < g.D(best))) best = c;
  };
  for (size_t k = 0; k < g.prims.size(); ++k) {
    if (done[k]) continue;
    const syno_prim& p = g.prims[k];
    switch (p.kind) {
      case SYNO_UNFOLD:
        if (b.K(p.out[0]) && !b.K(p.in[0]) && !b.K(p.in[1])) consider(p.in[1]);
        else if (!b.K(p.out[0]) && b.K(p.in[0]) != b.K(p.in[1])) consider(b.K(p.in[0]) ? p.in[1] : p.in[0]);
        break;
      case SYNO_MERGE:
        if (!b.K(p.in[0]) && b.K(p.out[0]) != b.K(p.out[1])) consider(b.K(p.out[0]) ? p.out[1] : p.out[0]);
        break;
      case SYNO_SPLIT:
        if (!b.K(p.out[0]) && b.K(p.in[0]) != b.K(p.in[1])) consider(b.K(p.in[0]) ? p.in[1] : p.in[0]);
        break;
      case SYNO_SHIFT:
        if (p.shift_by >= 0 && !b.K(p.shift_by) && (b.K(p.in[0]) || b.K(p.out[0]))) consider(p.shift_by);
        break;
      default: break;
    }
  }
  if (best >= 0) return best;
  for (int i = 0; i < g.n_out; ++i) consider(i);
  for (int c : g.reduce_coords) consider(c);
  return best;
}

struct TensorAxes {
  std::vector<int> coords;
  std::vector<int64_t> stride;
};

TensorAxes axes_of(const Graph& g, const std::vector<int>& coords) {
  TensorAxes t;
  t.coords = coords;
  t.stride.assign(coords.size(), 1);
  for (int i = (int)coords.size() - 2; i >= 0; --i) t.stride[i] = t.stride[i + 1] * g.D(coords[i + 1]);
  return t;
}

// Build the program that, for each element of `target` and each free point, yields the offsets
// into tensors `A` and `B`.  `forced_free` (forward pass only) fixes the free coordinates.
bool build_program(const Graph& g, const TensorAxes& target, const std::vector<int>* forced_free,
                   const TensorAxes& A, const TensorAxes& B, IndexProgram& out) {
  Builder b(g);
  std::memset(&out, 0, sizeof(out));
  // a coordinate value can be fixed by one target axis only
  for (size_t i = 0; i < target.coords.size(); ++i) {
    if (b.K(target.coords[i])) return false;
    b.set(target.coords[i]);
  }
  if (forced_free)
    for (int c : *forced_free) {
      if (b.K(c)) return false;
      b.set(c);
      b.free_slots.push_back(g.S(c));
    }
  std::vector<char> done(g.prims.size(), 0);
  for (;;) {
    bool progress = false;
    for (size_t k = 0; k < g.prims.size(); ++k)
      if (!done[k]) {
        const bool was = done[k];
        done[k] = step_prim(b, g.prims[k], &progress);
        if (done[k] != was) progress = true;
        if (b.failed) return false;
      }
    if (progress) continue;
    bool all = true;
    for (char d : done) all = all && d;
    for (int s = 0; s < g.n_slots; ++s) all = all && b.known[s];
    if (all) break;
    if (forced_free) return false;
    const int c = pick_free(b, done);
    if (c < 0) return false;
    b.set(c);
    b.free_slots.push_back(g.S(c));
  }
  if (!forced_free) std::reverse(b.free_slots.begin(), b.free_slots.end());   // first chosen varies fastest
  if (b.ops.size() > (size_t)kMaxOps || b.free_slots.size() > (size_t)kMaxAxes) return false;
  // split the ops into those that depend on the target only and the rest
  std::vector<char> dep(g.n_slots, 0);
  for (int s : b.free_slots) dep[s] = 1;
  std::vector<IndexOp> first, second;
  for (const IndexOp& o : b.ops) {
    bool d = dep[o.a] || (o.b >= 0 && dep[o.b]);
    if (o.d0 >= 0) dep[o.d0] = d;
    if (o.d1 >= 0) dep[o.d1] = d;
    (d ? second : first).push_back(o);
  }
  out.n_ops0 = (int32_t)first.size();
  out.n_ops = (int32_t)b.ops.size();
  int w = 0;
  for (const IndexOp& o : first) out.ops[w++] = o;
  for (const IndexOp& o : second) out.ops[w++] = o;
  out.n_tgt = (int32_t)target.coords.size();
  out.n_target = 1;
  for (int i = 0; i < out.n_tgt; ++i) {
    out.tgt[i] = AxisRef{g.S(target.coords[i]), (int32_t)g.D(target.coords[i]),
                         (int32_t)division_magic(g.D(target.coords[i]))};
    out.n_target = std::min<int64_t>(out.n_target * g.D(target.coords[i]), int64_t(1) << 40);  // (saturates: no overflow)
  }
  out.n_fre = (int32_t)b.free_slots.size();
  out.n_free = 1;
  for (int i = 0; i < out.n_fre; ++i) {
    out.fre[i] = AxisRef{b.free_slots[i], (int32_t)g.slot_dom[b.free_slots[i]],
                         (int32_t)division_magic(g.slot_dom[b.free_slots[i]])};
    out.n_free = std::min<int64_t>(out.n_free * g.slot_dom[b.free_slots[i]], int64_t(1) << 40);
  }
  out.n_a = (int32_t)A.coords.size();
  for (int i = 0; i < out.n_a; ++i)
    out.a[i] = AxisRef{g.S(A.coords[i]), (int32_t)g.D(A.coords[i]), (int32_t)A.stride[i]};
  out.n_b = (int32_t)B.coords.size();
  for (int i = 0; i < out.n_b; ++i)
    out.b[i] = AxisRef{g.S(B.coords[i]), (int32_t)g.D(B.coords[i]), (int32_t)B.stride[i]};
  return true;
}

// ---------------------------------------------------------------------------------------------
// Affine analysis of the forward index map and recognition of the convolution-like form
// ---------------------------------------------------------------------------------------------
struct Root {
  bool is_reduce = false;
  bool alive = true;
  int64_t size = 0;
  int64_t out_stride = 0;   // output iterators (and their digits): element stride in `out`
  int axis = -1;            // output iterators and their digits: value = (o_axis / div) % size
  int64_t div = 1;
};

struct Expr {
  std::map<int, int64_t> coef;   // root -> coefficient
  int64_t c = 0;
  int64_t wrap = 0;              // value is taken mod `wrap` when non-zero
  bool complex = false;
  bool pure() const { return !complex && wrap == 0; }
};

struct Check { Expr e; int64_t bound; };

Expr add(const Expr& x, int64_t kx, const Expr& y, int64_t ky, int64_t c) {
  Expr r;
  r.complex = !x.pure() || !y.pure();
  for (auto& t : x.coef) r.coef[t.first] += kx * t.second;
  for (auto& t : y.coef) r.coef[t.first] += ky * t.second;
  for (auto it = r.coef.begin(); it != r.coef.end();) it = it->second == 0 ? r.coef.erase(it) : std::next(it);
  r.c = kx * x.c + ky * y.c + c;
  return r;
}

bool same_affine(const Expr& a, const Expr& b) { return a.coef == b.coef && a.c == b.c; }

// Every coordinate as an affine expression of the iterators ("roots": output iterators, their Merge digits,
// Reduce iterators), plus the range tests the Unfolds impose.  False when the graph has an Expand (unless allowed:
// the expanded coordinate then simply influences nothing).
bool analyse(const Graph& g, std::vector<Root>& roots, std::vector<Expr>& e, std::vector<Check>& checks,
             bool allow_expand = false) {
  e.assign(g.n_slots, Expr());
  int n_reduce_seen = 0;
  for (int i = 0; i < g.n_out; ++i) {
    Root r; r.size = g.D(i); r.out_stride = g.out_stride[i]; r.axis = i;
    roots.push_back(r);
    e[g.S(i)].coef[(int)roots.size() - 1] = 1;
  }
  for (const syno_prim& p : g.prims) {
    switch (p.kind) {
      case SYNO_REDUCE: {
        Root r; r.is_reduce = true; r.size = p.param;
        r.axis = g.n_out + n_reduce_seen++;      // Reduce iterators count on after the output axes
        roots.push_back(r);
        e[g.S(p.out[0])].coef[(int)roots.size() - 1] = 1;
        break;
      }
      case SYNO_SHARE: break;
      case SYNO_EXPAND:
        if (!allow_expand) return false;
        break;
      case SYNO_MERGE: {
        const Expr& x = e[g.S(p.in[0])];
        if (!x.pure() || x.c != 0 || x.coef.size() != 1 || x.coef.begin()->second != 1) return false;
        const int r0 = x.coef.begin()->first;      // a bare iterator: refine it into two digits
        Root hi = roots[r0], lo = roots[r0];
        hi.size = roots[r0].size / p.param; hi.out_stride = roots[r0].out_stride * p.param;
        hi.div = roots[r0].div * p.param;
        lo.size = p.param;
        roots[r0].alive = false;
        roots.push_back(hi);
        e[g.S(p.out[0])].coef[(int)roots.size() - 1] = 1;
        roots.push_back(lo);
        e[g.S(p.out[1])].coef[(int)roots.size() - 1] = 1;
        break;
      }
      case SYNO_SPLIT:
        e[g.S(p.out[0])] = add(e[g.S(p.in[0])], g.D(p.in[1]), e[g.S(p.in[1])], 1, 0);
        break;
      case SYNO_STRIDE:
        e[g.S(p.out[0])] = add(e[g.S(p.in[0])], p.param, Expr(), 0, 0);
        break;
      case SYNO_SHIFT: {
        Expr by;
        if (p.shift_by >= 0) by = e[g.S(p.shift_by)];
        Expr r = add(e[g.S(p.in[0])], 1, by, p.shift_by >= 0 ? p.shift_coef : 0, p.param);
        r.wrap = g.D(p.in[0]);
        e[g.S(p.out[0])] = r;
        break;
      }
      case SYNO_UNFOLD: {
        Expr r = add(e[g.S(p.in[0])], 1, e[g.S(p.in[1])], 1, -(g.D(p.in[1]) / 2));
        checks.push_back(Check{r, g.D(p.in[0])});
        e[g.S(p.out[0])] = r;
        break;
      }
    }
  }
  return true;
}

bool recognise_conv(const Graph& g, ConvLike& cv) {
  std::vector<Root> roots;
  std::vector<Expr> e;
  std::vector<Check> checks;
  if (!analyse(g, roots, e, checks)) return false;
  // X is [n, channels, rows, columns]; a tensor without a row axis ([n, channels, columns]: a window over one long
  // axis) is the same with one row
  if (g.in_coords.size() != 4 && g.in_coords.size() != 3) return false;
  const Expr no_rows{};               // the constant 0
  const Expr* ax[4];
  int64_t ax_size[4];
  for (int i = 0, k = 0; i < 4; ++i) {
    if (i == 2 && g.in_coords.size() == 3) { ax[i] = &no_rows; ax_size[i] = 1; continue; }
    ax[i] = &e[g.S(g.in_coords[k])];
    ax_size[i] = g.D(g.in_coords[k]);
    ++k;
    if (ax[i]->complex) return false;
  }
  // roles
  enum { R_NONE, R_N, R_G, R_O, R_C, R_H, R_W, R_KH, R_KW };
  std::vector<int> role(roots.size(), R_NONE);
  std::memset(&cv, 0, sizeof(cv));
  cv.N = cv.G = cv.Og = cv.Cg = cv.Ho = cv.Wo = cv.KH = cv.KW = 1;
  cv.sh = cv.sw = 1;
  // axis 0: the batch iterator alone
  if (!ax[0]->pure() || ax[0]->c != 0 || ax[0]->coef.size() != 1) return false;
  {
    const int r = ax[0]->coef.begin()->first;
    if (ax[0]->coef.begin()->second != 1 || roots[r].is_reduce) return false;
    role[r] = R_N; cv.N = (int32_t)roots[r].size;
  }
  // axis 1: channel = Cg*g + c  |  c  |  g
  if (!ax[1]->pure() || ax[1]->c != 0 || ax[1]->coef.empty() || ax[1]->coef.size() > 2) return false;
  for (auto& t : ax[1]->coef) {
    if (role[t.first] != R_NONE) return false;
    if (roots[t.first].is_reduce) {
      if (t.second != 1 || cv.Cg != 1) return false;
      role[t.first] = R_C; cv.Cg = (int32_t)roots[t.first].size;
    } else {
      if (cv.G != 1) return false;
      role[t.first] = R_G; cv.G = (int32_t)roots[t.first].size;
    }
  }
  for (auto& t : ax[1]->coef)
    if (role[t.first] == R_G && t.second != cv.Cg) return false;
  if ((int64_t)cv.G * cv.Cg != g.D(g.in_coords[1])) return false;
  // axes 2, 3: s*h + kh - pad, zero outside; or (h + shift + coef*g) mod size
  for (int a = 2; a < 4; ++a) {
    const Expr& x = *ax[a];
    const int64_t size = ax_size[a];
    int32_t out_sz = 1, k_sz = 1, stride = 1, shift_g = 0;
    for (auto& t : x.coef) {
      const int r = t.first;
      if (role[r] == R_G) { if (!x.wrap) return false; shift_g = (int32_t)t.second; continue; }
      if (role[r] != R_NONE) return false;
      if (roots[r].is_reduce) {
        if (t.second != 1 || k_sz != 1 || x.wrap) return false;
        role[r] = a == 2 ? R_KH : R_KW; k_sz = (int32_t)roots[r].size;
      } else {
        if (t.second < 1 || out_sz != 1) return false;
        role[r] = a == 2 ? R_H : R_W; out_sz = (int32_t)roots[r].size; stride = (int32_t)t.second;
      }
    }
    if (x.wrap) {
      if (x.wrap != size || stride != 1 || out_sz != size) return false;
      (a == 2 ? cv.h_wrap : cv.w_wrap) = 1;
      (a == 2 ? cv.h_shift : cv.w_shift) = pos_mod(x.c, size);
      (a == 2 ? cv.h_shift_g : cv.w_shift_g) = pos_mod(shift_g, size);
    } else {
      if (x.c > 0) return false;
      (a == 2 ? cv.ph : cv.pw) = (int32_t)(-x.c);
    }
    (a == 2 ? cv.Ho : cv.Wo) = out_sz;
    (a == 2 ? cv.KH : cv.KW) = k_sz;
    (a == 2 ? cv.sh : cv.sw) = stride;
    (a == 2 ? cv.Hi : cv.Wi) = (int32_t)size;
    // Without a window the map must stay inside the axis by itself; with one the Unfold's test guards it.
    const int64_t lo = x.c, hi = x.c + (int64_t)stride * (out_sz - 1) + (k_sz - 1);
    if (!x.wrap && k_sz == 1 && (lo < 0 || hi >= size)) return false;
  }
  // every range test must be exactly "this X axis lies inside its size"
  for (const Check& c : checks) {
    bool ok = false;
    for (int a = 2; a < 4; ++a)
      if (!ax[a]->wrap && same_affine(c.e, *ax[a]) && c.bound == ax_size[a]) ok = true;
    if (!ok) return false;
  }
  // weight axes: one bare iterator each
  std::vector<int64_t> wstride(g.w_coords.size(), 1);
  for (int i = (int)g.w_coords.size() - 2; i >= 0; --i) wstride[i] = wstride[i + 1] * g.D(g.w_coords[i + 1]);
  std::vector<char> in_w(roots.size(), 0);
  for (size_t i = 0; i < g.w_coords.size(); ++i) {
    const Expr& x = e[g.S(g.w_coords[i])];
    if (!x.pure() || x.c != 0 || x.coef.size() != 1 || x.coef.begin()->second != 1) return false;
    const int r = x.coef.begin()->first;
    if (in_w[r]) return false;
    in_w[r] = 1;
    if (role[r] == R_NONE) {
      if (roots[r].is_reduce || cv.Og != 1) return false;
      role[r] = R_O; cv.Og = (int32_t)roots[r].size;
    }
    const int32_t s = (int32_t)wstride[i];
    switch (role[r]) {
      case R_G: cv.ws_g = s; break;
      case R_O: cv.ws_o = s; break;
      case R_C: cv.ws_c = s; break;
      case R_KH: cv.ws_kh = s; break;
      case R_KW: cv.ws_kw = s; break;
      default: return false;      // batch or spatial iterators do not index the weight here
    }
  }
  // every live iterator has a role; reduce iterators must reach the weight (else it is a plain sum)
  for (size_t r = 0; r < roots.size(); ++r) {
    if (!roots[r].alive) continue;
    if (role[r] == R_NONE) return false;
    if (roots[r].is_reduce && !in_w[r]) return false;
    if (role[r] == R_G && !in_w[r] && roots[r].size > 1) return false;
  }
  // the output must be laid out [N, G*Og, Ho, Wo]
  int64_t expect[9] = {};
  expect[R_W] = 1; expect[R_H] = cv.Wo; expect[R_O] = (int64_t)cv.Ho * cv.Wo;
  expect[R_G] = expect[R_O] * cv.Og; expect[R_N] = expect[R_G] * cv.G;
  for (size_t r = 0; r < roots.size(); ++r) {
    if (!roots[r].alive || roots[r].is_reduce) continue;
    if (roots[r].size > 1 && roots[r].out_stride != expect[role[r]]) return false;
  }
  return true;
}

// The window form whose window iterator is Shared with the weight but not Reduced (first stage of Operator 1,
// Fig. 7): out laid out [n,d,g,k,h,w], X = [n, Cg*g+c, h, w+k-pw], the weight indexed by bare d, g, c, k.
bool recognise_share_window(const Graph& g, ShareWindow& sw) {
  std::vector<Root> roots;
  std::vector<Expr> e;
  std::vector<Check> checks;
  if (!analyse(g, roots, e, checks)) return false;
  if (g.in_coords.size() != 4 || checks.size() != 1) return false;
  const Expr* ax[4];
  for (int i = 0; i < 4; ++i) {
    ax[i] = &e[g.S(g.in_coords[i])];
    if (!ax[i]->pure()) return false;
  }
  enum { R_NONE, R_N, R_D, R_G, R_K, R_H, R_W, R_C };
  std::vector<int> role(roots.size(), R_NONE);
  std::memset(&sw, 0, sizeof(sw));
  sw.N = sw.D = sw.G = sw.K = sw.H = sw.W = sw.Cg = 1;
  auto bare_output = [&](const Expr& x, int r_role, int32_t& size) {
    if (x.c != 0 || x.coef.size() != 1 || x.coef.begin()->second != 1) return false;
    const int r = x.coef.begin()->first;
    if (roots[r].is_reduce || role[r] != R_NONE) return false;
    role[r] = r_role; size = (int32_t)roots[r].size;
    return true;
  };
  if (!bare_output(*ax[0], R_N, sw.N) || !bare_output(*ax[2], R_H, sw.H)) return false;
  if (sw.H != g.D(g.in_coords[2])) return false;
  // channel = Cg*g + c  |  c
  if (ax[1]->c != 0 || ax[1]->coef.empty() || ax[1]->coef.size() > 2) return false;
  for (auto& t : ax[1]->coef) {
    if (role[t.first] != R_NONE) return false;
    if (roots[t.first].is_reduce) {
      if (t.second != 1 || sw.Cg != 1) return false;
      role[t.first] = R_C; sw.Cg = (int32_t)roots[t.first].size;
    } else {
      if (sw.G != 1) return false;
      role[t.first] = R_G; sw.G = (int32_t)roots[t.first].size;
    }
  }
  for (auto& t : ax[1]->coef)
    if (role[t.first] == R_G && t.second != sw.Cg) return false;
  if ((int64_t)sw.G * sw.Cg != g.D(g.in_coords[1])) return false;
  // column = w + k - pw: two output iterators; the one whose size is the axis is w, the other the window
  if (ax[3]->coef.size() != 2 || ax[3]->c > 0) return false;
  sw.pw = (int32_t)(-ax[3]->c);
  const int64_t Wi = g.D(g.in_coords[3]);
  int rw = -1, rk = -1;
  for (auto& t : ax[3]->coef) {
    if (t.second != 1 || roots[t.first].is_reduce || role[t.first] != R_NONE) return false;
    if (roots[t.first].size == Wi && rw < 0) rw = t.first; else rk = t.first;
  }
  if (rw < 0 || rk < 0) return false;
  role[rw] = R_W; sw.W = (int32_t)roots[rw].size;
  role[rk] = R_K; sw.K = (int32_t)roots[rk].size;
  if (sw.pw != sw.K / 2 || sw.K < 2) return false;
  if (!same_affine(checks[0].e, *ax[3]) || checks[0].bound != Wi) return false;
  // weight axes: one bare iterator each; every iterator of extent > 1 other than n, h, w must index it
  std::vector<int64_t> wstride(g.w_coords.size(), 1);
  for (int i = (int)g.w_coords.size() - 2; i >= 0; --i) wstride[i] = wstride[i + 1] * g.D(g.w_coords[i + 1]);
  std::vector<char> in_w(roots.size(), 0);
  for (size_t i = 0; i < g.w_coords.size(); ++i) {
    const Expr& x = e[g.S(g.w_coords[i])];
    if (!x.pure() || x.c != 0 || x.coef.size() != 1 || x.coef.begin()->second != 1) return false;
    const int r = x.coef.begin()->first;
    if (in_w[r]) return false;
    in_w[r] = 1;
    if (role[r] == R_NONE) {
      if (roots[r].is_reduce || sw.D != 1) return false;
      role[r] = R_D; sw.D = (int32_t)roots[r].size;
    }
    const int32_t s = (int32_t)wstride[i];
    switch (role[r]) {
      case R_D: sw.ws_d = s; break;
      case R_G: sw.ws_g = s; break;
      case R_C: sw.ws_c = s; break;
      case R_K: sw.ws_k = s; break;
      default: return false;
    }
  }
  for (size_t r = 0; r < roots.size(); ++r) {
    if (!roots[r].alive) continue;
    if (role[r] == R_NONE) return false;
    const bool needs_w = role[r] == R_D || role[r] == R_G || role[r] == R_C || role[r] == R_K;
    if (needs_w && !in_w[r] && roots[r].size > 1) return false;
  }
  // the output must be laid out [N, D, G, K, H, W]
  int64_t expect[8] = {};
  expect[R_W] = 1; expect[R_H] = sw.W; expect[R_K] = (int64_t)sw.H * sw.W; expect[R_G] = expect[R_K] * sw.K;
  expect[R_D] = expect[R_G] * sw.G; expect[R_N] = expect[R_D] * sw.D;
  for (size_t r = 0; r < roots.size(); ++r) {
    if (!roots[r].alive || roots[r].is_reduce) continue;
    if (roots[r].size > 1 && roots[r].out_stride != expect[role[r]]) return false;
  }
  return true;
}

// out[i,j] = sum_k X[i,k] * W[k,j] (Table 2's matrix multiplication): two output iterators, one Reduce Shared
// between X's inner axis and W's outer axis, nothing else.
bool recognise_matmul(const Graph& g, int64_t& M, int64_t& K, int64_t& N) {
  std::vector<Root> roots;
  std::vector<Expr> e;
  std::vector<Check> checks;
  if (!analyse(g, roots, e, checks)) return false;
  if (g.n_out != 2 || g.in_coords.size() != 2 || g.w_coords.size() != 2 || !checks.empty()) return false;
  int alive = 0;
  for (const Root& r : roots) alive += r.alive ? 1 : 0;
  if (alive != 3 || roots.size() != 3) return false;
  auto bare = [&](int coord) {
    const Expr& x = e[g.S(coord)];
    if (!x.pure() || x.c != 0 || x.coef.size() != 1 || x.coef.begin()->second != 1) return -1;
    return x.coef.begin()->first;
  };
  const int xi = bare(g.in_coords[0]), xk = bare(g.in_coords[1]);
  const int wk = bare(g.w_coords[0]), wj = bare(g.w_coords[1]);
  if (xi != 0 || wj != 1 || xk != 2 || wk != 2 || !roots[2].is_reduce) return false;
  M = roots[0].size; N = roots[1].size; K = roots[2].size;
  return true;
}

// Graphs without range tests and with at most a few sum points per output: the separable form of plan.h
// (ViewStream).
constexpr int64_t kMaxViewSumPoints = 64;
bool recognise_view(const Graph& g, ViewStream& vs) {
  if (g.n_out < 1 || (int)g.reduce_coords.size() > kMaxAxes) return false;
  int64_t sum_points = 1;
  for (int c : g.reduce_coords) sum_points *= g.D(c);
  if (sum_points > kMaxViewSumPoints) return false;
  std::vector<Root> roots;
  std::vector<Expr> e;
  std::vector<Check> checks;
  if (!analyse(g, roots, e, checks, true) || !checks.empty()) return false;
  std::memset(&vs, 0, sizeof(vs));
  vs.n_axes = g.n_out;
  for (int i = 0; i < g.n_out; ++i) vs.size[i] = (int32_t)g.D(i);
  vs.n_red = (int32_t)g.reduce_coords.size();
  for (int j = 0; j < vs.n_red; ++j) vs.size[g.n_out + j] = (int32_t)g.D(g.reduce_coords[j]);
  auto add_tensor = [&](const std::vector<int>& coords, int tensor) {
    std::vector<int64_t> stride(coords.size(), 1);
    for (int i = (int)coords.size() - 2; i >= 0; --i) stride[i] = stride[i + 1] * g.D(coords[i + 1]);
    for (size_t j = 0; j < coords.size(); ++j) {
      const Expr& x = e[g.S(coords[j])];
      if (x.complex || vs.n_groups >= kMaxViewGroups) return false;
      ViewGroup& grp = vs.group[vs.n_groups];
      grp.tensor = tensor; grp.stride = (int32_t)stride[j]; grp.wrap = (int32_t)x.wrap; grp.axis = 0;
      grp.c = (int32_t)(x.wrap ? pos_mod(x.c, x.wrap) : x.c);
      int one_axis = -1;
      for (auto& t : x.coef) {
        const Root& r = roots[t.first];
        if (r.axis < 0 || vs.n_terms >= kMaxViewTerms) return false;
        if (one_axis >= 0 && one_axis != r.axis && x.wrap) return false;     // a wrap over two output axes
        one_axis = r.axis;
        if (x.wrap && t.second < 0) return false;
        vs.term[vs.n_terms++] = ViewTerm{vs.n_groups, r.axis, (int32_t)r.div, (int32_t)r.size, (int32_t)t.second};
      }
      if (one_axis >= 0) grp.axis = one_axis;
      // without a wrap the value must stay inside the axis by itself
      if (!x.wrap) {
        int64_t lo = x.c, hi = x.c;
        for (auto& t : x.coef) (t.second < 0 ? lo : hi) += t.second * (roots[t.first].size - 1);
        if (lo < 0 || hi >= g.D(coords[j])) return false;
      }
      ++vs.n_groups;
    }
    return true;
  };
  if (!add_tensor(g.in_coords, 0) || !add_tensor(g.w_coords, 1)) return false;
  // Backward-data as a scatter needs the map from outputs to X elements to be one-to-one and onto.  Split, Merge
  // and Shift are bijections of coordinates and Share copies one; what is left to rule out is a copy that comes
  // back into X (a diagonal) or an iterator that only reaches the weight.  Checked on the record itself: every X
  // axis must enumerate its own range in mixed radix (its terms, by rising coefficient: 1, s1, s1*s2, ... with
  // the sizes' product equal to the axis; a wrap then only rotates that range), no digit may feed two X axes, and
  // X must have as many elements as there are outputs, so that no digit is left out.
  int64_t x_elems = 1, out_elems = 1;
  for (int c : g.in_coords) x_elems *= g.D(c);
  for (int i = 0; i < g.n_out; ++i) out_elems *= g.D(i);
  bool one = vs.n_red == 0 && x_elems == out_elems;
  for (const syno_prim& p : g.prims)
    if (p.kind != SYNO_SPLIT && p.kind != SYNO_MERGE && p.kind != SYNO_SHIFT && p.kind != SYNO_SHARE) one = false;
  std::vector<std::array<int32_t, 3>> seen;      // digits (axis, div, size) already feeding an X axis
  for (int gi = 0; one && gi < (int)g.in_coords.size(); ++gi) {
    std::vector<std::pair<int64_t, int64_t>> digits;   // (coefficient, size)
    for (int t = 0; t < vs.n_terms; ++t) {
      const ViewTerm& tm = vs.term[t];
      if (tm.group != gi) continue;
      const std::array<int32_t, 3> key = {tm.axis, tm.div, tm.size};
      if (std::find(seen.begin(), seen.end(), key) != seen.end()) one = false;
      seen.push_back(key);
      digits.emplace_back(tm.coef, tm.size);
    }
    std::sort(digits.begin(), digits.end());
    int64_t expect = 1;
    for (auto& dg : digits) {
      if (dg.first != expect) one = false;
      expect *= dg.second;
    }
    if (expect != g.D(g.in_coords[gi])) one = false;
  }
  vs.one_to_one = one ? 1 : 0;
  return true;
}

// The width to fold the N contiguous output columns of a matrix product into image rows of: the 1x1
// convolution does not couple pixels, so any factorisation N = rows * width is the same contraction; widths
// near the ones the contraction kernels are tuned on are preferred.  0 when N has no usable divisor.
int64_t fold_width(int64_t N) {
  if (N <= 64) return N >= 4 ? N : 0;
  int64_t best = 0;
  for (int64_t w = 64; w >= 7; --w)
    if (N % w == 0 && (best == 0 || std::llabs(w - 56) < std::llabs(best - 56))) best = w;
  return best;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// Materialised reduction (code-generation section of the paper).  FLOPs are the output iterators times all Reduces;
// a Reduce evaluated below a one-to-many primitive (Unfold, Expand) is repeated for every copy.  Lowering a Reduce
// only needs the primitives that lie between it and the tensors; evaluating exactly those first and storing
// their result removes the repetition.  For every Reduce the pass takes that upward closure, makes the
// coordinates entering it from below (and the tensor axes it does not touch) the axes of the stored tensor Z, and
// keeps the cut with the fewest multiply-adds if it beats the single loop nest; the rest of the graph is cut
// again the same way.
// ---------------------------------------------------------------------------------------------
namespace {

// weight_on_top: index into `whole`'s weights (0 = win, 1.. = the further ones) of the weight the top stage takes, -1: none
bool cut_once(const OwnedDesc& whole, OwnedDesc& top, OwnedDesc& bottom, int& weight_on_top) {
  const syno_desc d = whole.view();
  Graph g;
  if (parse_graph(&d, g, nullptr) != SYNO_OK) return false;
  const int n = (int)g.prims.size();
  for (const syno_prim& p : g.prims)
    if (p.kind == SYNO_SHIFT && p.shift_by >= 0) return false;   // a coordinate read without being consumed: not cut
  double out_points = 1, all_red = 1;
  for (int i = 0; i < g.n_out; ++i) out_points *= (double)g.D(i);
  for (int c : g.reduce_coords) all_red *= (double)g.D(c);
  const double before = out_points * all_red;
  // the weights `whole` still carries (a stage cut off earlier may have taken the first one: then win is empty and
  // there is no weight 0)
  std::vector<const std::vector<int>*> weights;
  const bool has_w0 = !whole.weight_ids.empty() && whole.weight_ids[0] >= 0;
  weights.push_back(&g.w_coords);
  for (const auto& w : g.more_w) weights.push_back(&w);
  std::vector<int> weight_of(kMaxCoordId, -1);        // coordinate -> the weight it indexes
  for (size_t wi = 0; wi < weights.size(); ++wi)
    for (int c : *weights[wi]) weight_of[c] = (int)wi;
  std::vector<int> producer(kMaxCoordId, -1);
  for (int k = 0; k < n; ++k)
    for (int t = 0; t < arity_out(g.prims[k].kind); ++t) producer[g.prims[k].out[t]] = k;

  double best = before;
  std::vector<char> best_c;
  std::vector<int> best_z;
  int best_w = -1;
  for (int r = 0; r < n; ++r) {
    if (g.prims[r].kind != SYNO_REDUCE) continue;
    std::vector<char> in_c(n, 0), coord_c(kMaxCoordId, 0);
    in_c[r] = 1; coord_c[g.prims[r].out[0]] = 1;
    auto close = [&]() {           // every primitive that consumes a closure coordinate joins, with what it produces
      for (int k = 0; k < n; ++k) {
        if (in_c[k]) continue;
        const syno_prim& p = g.prims[k];
        bool touches = false;
        for (int t = 0; t < arity_in(p.kind); ++t) touches |= coord_c[p.in[t]] != 0;
        if (!touches) continue;
        in_c[k] = 1;
        for (int t = 0; t < arity_out(p.kind); ++t) coord_c[p.out[t]] = 1;
      }
    };
    close();
    auto touched = [&]() {         // the weight the closure reaches: -1 none, -2 more than one
      int w = -1;
      for (int c = 0; c < kMaxCoordId; ++c)
        if (coord_c[c] && weight_of[c] >= 0) w = (w < 0 || w == weight_of[c]) ? weight_of[c] : -2;
      return w;
    };
    int on_w = touched();
    if (on_w == -2 || (on_w == 0 && !has_w0)) continue;
    if (on_w >= 0 && weights.size() > 1) {
      // several weights: the stage that multiplies with this weight also takes the Shares that hand the weight its
      // other coordinates, when their second copy goes on towards the data (not straight into another weight), and
      // with them whatever consumes that copy
      bool grown = true;
      while (grown) {
        grown = false;
        for (int c : *weights[on_w]) {
          if (coord_c[c]) continue;
          const int k = producer[c];
          if (k < 0 || g.prims[k].kind != SYNO_SHARE) continue;
          const int other = g.prims[k].out[0] == c ? g.prims[k].out[1] : g.prims[k].out[0];
          if (weight_of[other] >= 0) continue;
          in_c[k] = 1; coord_c[g.prims[k].out[0]] = coord_c[g.prims[k].out[1]] = 1;
          close();
          grown = true;
        }
      }
      if (touched() != on_w) continue;
    }
    double red_c = 1;
    for (int k = 0; k < n; ++k)
      if (in_c[k] && g.prims[k].kind == SYNO_REDUCE) red_c *= (double)g.prims[k].param;
    // axes of Z, in the order of X's axes: an axis the closure does not produce passes through, one it produces
    // is replaced by the coordinates that enter the closure below it
    std::vector<int> z;
    std::vector<char> seen(kMaxCoordId, 0);
    auto add = [&](int c) { if (!seen[c]) { seen[c] = 1; z.push_back(c); } };
    std::vector<int> stack;
    auto below = [&](int axis) {
      stack.assign(1, axis);
      while (!stack.empty()) {
        const int c = stack.back(); stack.pop_back();
        if (!coord_c[c]) { add(c); continue; }
        const int k = producer[c];
        if (k < 0) continue;
        const syno_prim& p = g.prims[k];
        for (int t = arity_in(p.kind) - 1; t >= 0; --t) stack.push_back(p.in[t]);
      }
    };
    for (int c : g.in_coords) below(c);
    const size_t n_from_x = z.size();
    if (on_w >= 0) for (int c : *weights[on_w]) below(c);
    // Z's layout is the pass's to choose.  Keep X's order, but in the arrangement the lowered forms look for: the
    // leading axes of X that pass through untouched (batch), then the iterators that only the stage's weight brings
    // (its output channels), then the other coordinates that are not image axes (channel digits, window iterators),
    // then the image axes (coordinates that an Unfold anywhere in the graph slides a window over).
    {
      std::vector<char> spatial(kMaxCoordId, 0);
      for (const syno_prim& q : g.prims)
        if (q.kind == SYNO_UNFOLD) spatial[q.in[0]] = spatial[q.out[0]] = 1;
      for (bool grown = true; grown;) {      // ... or over the coarse part of which it is (Split, Merge, Stride, Shift)
        grown = false;
        for (const syno_prim& q : g.prims)
          if (q.kind == SYNO_SPLIT || q.kind == SYNO_MERGE || q.kind == SYNO_STRIDE || q.kind == SYNO_SHIFT)
            if (spatial[q.in[0]] != spatial[q.out[0]]) { spatial[q.in[0]] = spatial[q.out[0]] = 1; grown = true; }
      }
      std::vector<int> lead, from_w, other, image;
      bool leading = true;
      for (size_t i = 0; i < z.size(); ++i) {
        const int c = z[i];
        const bool untouched_axis = i < n_from_x && std::find(g.in_coords.begin(), g.in_coords.end(), c) != g.in_coords.end();
        if (i >= n_from_x) { from_w.push_back(c); continue; }
        if (spatial[c]) { image.push_back(c); leading = false; continue; }
        if (leading && untouched_axis) lead.push_back(c);
        else { other.push_back(c); leading = false; }
      }
      z = lead;
      z.insert(z.end(), from_w.begin(), from_w.end());
      z.insert(z.end(), other.begin(), other.end());
      z.insert(z.end(), image.begin(), image.end());
    }
    // every coordinate entering the closure from below must have been found (it is, through X or W, unless the
    // closure ends in an Expand, which has no top side)
    bool complete = true;
    for (int k = 0; k < n && complete; ++k)
      if (in_c[k])
        for (int t = 0; t < arity_in(g.prims[k].kind); ++t)
          if (!coord_c[g.prims[k].in[t]] && !seen[g.prims[k].in[t]]) complete = false;
    if (!complete || z.empty() || (int)z.size() > kMaxAxes) continue;
    double z_points = 1;
    for (int c : z) z_points *= (double)g.D(c);
    if (z_points > (double)kMaxElems) continue;
    const double after = z_points * red_c + out_points * (all_red / red_c);
    if (after < best) { best = after; best_c = in_c; best_z = z; best_w = on_w; }
  }
  if (best_c.empty()) return false;

  // top stage: Z's axes are its output iterators 0..nz-1, the closure's primitives follow with fresh ids
  std::vector<int> remap(kMaxCoordId, -1);
  top = OwnedDesc{};
  int next = 0;
  for (int c : best_z) {
    remap[c] = next++;
    top.dims.push_back(syno_dim{nullptr, g.D(c)});
  }
  for (int k = 0; k < n; ++k) {
    if (!best_c[k]) continue;
    syno_prim p = g.prims[k];
    for (int t = 0; t < arity_in(p.kind); ++t) p.in[t] = remap[p.in[t]];
    for (int t = 0; t < arity_out(p.kind); ++t) { remap[p.out[t]] = next; p.out[t] = next++; }
    top.prims.push_back(p);
  }
  if (next > kMaxCoordId) return false;
  for (int c : g.in_coords) top.xin.push_back(remap[c]);
  if (best_w >= 0) for (int c : *weights[best_w]) top.win.push_back(remap[c]);
  top.weight_ids.assign(1, best_w >= 0 ? whole.weight_ids[best_w] : -1);
  top.in_dtype = whole.in_dtype; top.out_dtype = whole.in_dtype;
  top.opt = whole.opt; top.has_opt = whole.has_opt;
  // bottom stage: the rest of the graph with its ids, reading Z; it keeps the other weights
  bottom = OwnedDesc{};
  bottom.dims = whole.dims;
  for (int k = 0; k < n; ++k) if (!best_c[k]) bottom.prims.push_back(g.prims[k]);
  bottom.xin.assign(best_z.begin(), best_z.end());
  bottom.weight_ids.assign(1, -1);
  for (size_t wi = 0; wi < weights.size(); ++wi) {
    if ((int)wi == best_w || (wi == 0 && !has_w0)) continue;
    if (bottom.weight_ids[0] < 0 && bottom.win.empty() && bottom.more_ranks.empty()) {
      bottom.win.assign(weights[wi]->begin(), weights[wi]->end());
      bottom.weight_ids[0] = whole.weight_ids[wi];
    } else {
      bottom.more_ranks.push_back((int32_t)weights[wi]->size());
      bottom.more_flat.insert(bottom.more_flat.end(), weights[wi]->begin(), weights[wi]->end());
      bottom.weight_ids.push_back(whole.weight_ids[wi]);
    }
  }
  bottom.in_dtype = whole.in_dtype; bottom.out_dtype = whole.out_dtype;
  bottom.opt = whole.opt; bottom.has_opt = whole.has_opt;
  weight_on_top = best_w;
  // both halves must be valid graphs by themselves
  Graph gt, gb;
  const syno_desc dt = top.view(), db = bottom.view();
  return parse_graph(&dt, gt, nullptr) == SYNO_OK && parse_graph(&db, gb, nullptr) == SYNO_OK;
}

}  // namespace

syno_status materialise(const syno_desc* desc, std::vector<OwnedDesc>& stages, std::vector<int32_t>& stage_weight) {
  Graph g;
  const syno_status st = parse_graph(desc, g, nullptr);
  if (st != SYNO_OK) return st;
  OwnedDesc cur;
  cur.dims.assign(desc->out_dims, desc->out_dims + desc->n_out);
  cur.prims.assign(desc->prims, desc->prims + desc->n_prim);
  cur.xin.assign(desc->input_coords, desc->input_coords + desc->n_in);
  cur.win.assign(desc->weight_coords, desc->weight_coords + desc->n_w);
  cur.weight_ids.assign(1, 0);
  for (size_t k = 0; k < g.more_w.size(); ++k) {
    cur.more_ranks.push_back((int32_t)g.more_w[k].size());
    cur.more_flat.insert(cur.more_flat.end(), g.more_w[k].begin(), g.more_w[k].end());
    cur.weight_ids.push_back((int32_t)k + 1);
  }
  cur.in_dtype = desc->in_dtype; cur.out_dtype = desc->out_dtype;
  if (desc->options) { cur.opt = *desc->options; cur.has_opt = true; }
  stages.clear();
  stage_weight.clear();
  while (stages.size() + 1 < 8) {
    OwnedDesc top, bottom;
    int on_top = -1;
    if (!cut_once(cur, top, bottom, on_top)) break;
    stage_weight.push_back(top.weight_ids[0]);
    stages.push_back(std::move(top));
    cur = std::move(bottom);
  }
  // what is left is the last stage; it may keep one weight
  if (!cur.more_ranks.empty()) return SYNO_ERR_UNSUPPORTED;      // several weights that did not come apart
  stage_weight.push_back(cur.weight_ids[0]);
  stages.push_back(std::move(cur));
  return SYNO_OK;
}

// ---------------------------------------------------------------------------------------------
namespace {
// Adjacent axes of X that are both plain Reduce iterators Shared with the weight, whose weight copies are adjacent
// axes of W in the same order, are one iterator of the product size as far as memory goes (row-major layouts on
// both sides).  So are the two halves of a Merge that lie side by side in X.  Returns the descriptor with every such
// pair fused (and its ids renumbered), or false when there is none.  The tensors' bytes are the same, so a lowered form recognised on the fused graph serves the original.
bool fuse_reduced_axes(const syno_desc& d, OwnedDesc& out) {
  std::vector<syno_prim> P(d.prims, d.prims + d.n_prim);
  std::vector<int32_t> xin(d.input_coords, d.input_coords + d.n_in), win(d.weight_coords, d.weight_coords + d.n_w);
  bool any = false;
  for (bool again = true; again;) {
    again = false;
    auto producer = [&](int c) {
      for (size_t k = 0; k < P.size(); ++k)
        for (int t = 0; t < arity_out(P[k].kind); ++t)
          if (P[k].out[t] == c) return (int)k;
      return -1;
    };
    // the Share that hands `a` to X and its other copy to W, fed by a Reduce directly: (share, reduce, weight copy)
    auto shared_reduce = [&](int a, int& sh, int& rd, int& b) {
      sh = producer(a);
      if (sh < 0 || P[sh].kind != SYNO_SHARE) return false;
      rd = producer(P[sh].in[0]);
      if (rd < 0 || P[rd].kind != SYNO_REDUCE) return false;
      b = P[sh].out[0] == a ? P[sh].out[1] : P[sh].out[0];
      return std::find(win.begin(), win.end(), b) != win.end();
    };
    // Two adjacent axes of X that are the quotient and the remainder of one Merge are, in memory, the axis the Merge
    // divided (offset q*B + r): X takes that coordinate directly and the Merge goes.  This is how a window over a
    // flattened pair of axes (an Unfold below a Merge) becomes a window over one long axis.
    for (size_t i = 0; i + 1 < xin.size() && !again; ++i) {
      const int mk = producer(xin[i]);
      if (mk < 0 || P[mk].kind != SYNO_MERGE || P[mk].out[0] != xin[i] || P[mk].out[1] != xin[i + 1]) continue;
      bool read_elsewhere = false;
      for (const syno_prim& q : P)
        if (q.kind == SYNO_SHIFT && q.shift_by >= 0) read_elsewhere |= q.shift_by == xin[i] || q.shift_by == xin[i + 1];
      if (read_elsewhere) continue;
      xin[i] = P[mk].in[0];
      xin.erase(xin.begin() + i + 1);
      P.erase(P.begin() + mk);
      again = any = true;
    }
    for (size_t i = 0; i + 1 < xin.size() && !again; ++i) {
      int s1, r1, b1, s2, r2, b2;
      if (!shared_reduce(xin[i], s1, r1, b1) || !shared_reduce(xin[i + 1], s2, r2, b2)) continue;
      const size_t p1 = std::find(win.begin(), win.end(), b1) - win.begin();
      if (p1 + 1 >= win.size() || win[p1 + 1] != b2) continue;
      bool read_elsewhere = false;          // (a Shift may read a coordinate without consuming it)
      for (const syno_prim& q : P)
        if (q.kind == SYNO_SHIFT && q.shift_by >= 0)
          for (int c : {xin[i], xin[i + 1], b1, b2, P[s1].in[0], P[s2].in[0]}) read_elsewhere |= q.shift_by == c;
      if (read_elsewhere) continue;
      P[r1].param *= P[r2].param;
      xin.erase(xin.begin() + i + 1);
      win.erase(win.begin() + p1 + 1);
      for (int k : {std::max(s2, r2), std::min(s2, r2)}) P.erase(P.begin() + k);
      again = any = true;
    }
  }
  if (!any) return false;
  // renumber: output iterators keep their ids, every other coordinate gets the next free one in definition order
  std::vector<int> remap(kMaxCoordId, -1);
  int next = d.n_out;
  for (int i = 0; i < d.n_out; ++i) remap[i] = i;
  out = OwnedDesc{};
  out.dims.assign(d.out_dims, d.out_dims + d.n_out);
  for (syno_prim q : P) {
    for (int t = 0; t < arity_in(q.kind); ++t) q.in[t] = remap[q.in[t]];
    if (q.kind == SYNO_SHIFT && q.shift_by >= 0) q.shift_by = remap[q.shift_by];
    for (int t = 0; t < arity_out(q.kind); ++t) { remap[q.out[t]] = next; q.out[t] = next++; }
    out.prims.push_back(q);
  }
  for (int c : xin) out.xin.push_back(remap[c]);
  for (int c : win) out.win.push_back(remap[c]);
  out.in_dtype = d.in_dtype; out.out_dtype = d.out_dtype;
  return true;
}
}  // namespace

syno_status build_plan(const syno_desc* desc, syno_plan* plan, std::string* why) {
  if (desc->options) plan->opt = *desc->options;
  const int policy = plan->opt.kernel_policy;
  Graph g;
  syno_status st = parse_graph(desc, g, why);
  if (st != SYNO_OK) return st;
  auto unsupported = [&](const char* m) { if (why) *why = m; return SYNO_ERR_UNSUPPORTED; };
  if (!g.more_w.empty()) return unsupported("an operator with several weights is evaluated in stages");

  plan->in_dtype = desc->in_dtype;
  plan->out_dtype = desc->out_dtype;
  plan->out_rank = g.n_out;
  plan->out_elems = 1;
  for (int i = 0; i < g.n_out; ++i) { plan->out_shape[i] = g.D(i); plan->out_elems *= g.D(i); }
  plan->x_rank = (int32_t)g.in_coords.size();
  plan->x_elems = 1;
  for (int i = 0; i < plan->x_rank; ++i) { plan->x_shape[i] = g.D(g.in_coords[i]); plan->x_elems *= plan->x_shape[i]; }
  plan->w_rank = (int32_t)g.w_coords.size();
  plan->w_elems = 1;
  for (int i = 0; i < plan->w_rank; ++i) { plan->w_shape[i] = g.D(g.w_coords[i]); plan->w_elems *= plan->w_shape[i]; }
  plan->n_reduce = 1;
  for (int c : g.reduce_coords) plan->n_reduce *= g.D(c);
  if (plan->out_elems > kMaxElems || plan->x_elems > kMaxElems || plan->w_elems > kMaxElems ||
      plan->n_reduce > kMaxElems)
    return unsupported("a tensor has more than 2^31-1 elements");
  // Shift offsets are reduced mod N on the host; the kernel's sum i + s + coef*v must fit 32 bits.
  for (const syno_prim& p : g.prims)
    if (p.kind == SYNO_SHIFT) {
      const int64_t N = g.D(p.in[0]), by = p.shift_by >= 0 ? g.D(p.shift_by) : 1;
      if (2 * N + N * by > kMaxElems) return unsupported("Shift offset range too large");
    }

  std::vector<int> outs(g.n_out);
  for (int i = 0; i < g.n_out; ++i) outs[i] = i;
  const TensorAxes O = axes_of(g, outs), X = axes_of(g, g.in_coords), W = axes_of(g, g.w_coords);
  if (!build_program(g, O, &g.reduce_coords, X, W, plan->prog[SYNO_FWD]))
    return unsupported("forward index map could not be lowered");
  if (!build_program(g, X, nullptr, O, W, plan->prog[SYNO_BWD_DATA]))
    return unsupported("backward-data index map could not be inverted");
  if (!build_program(g, W, nullptr, O, X, plan->prog[SYNO_BWD_WEIGHT]))
    return unsupported("backward-weight index map could not be inverted");

  for (int which = 0; which < 3; ++which)   // the kernels decode flat target and sum-point indices in 32 bits
    if (plan->prog[which].n_target > kMaxElems || plan->prog[which].n_free > kMaxElems)
      return unsupported("more than 2^31-1 sum points per element in one of the passes");

  plan->conv_like = recognise_conv(g, plan->conv);
  if (!plan->conv_like) {      // several reduced channel-like axes side by side (a stage cut off by the pass), or the
                               // two halves of a Merge side by side (a window over flattened axes): one axis
    OwnedDesc fused;
    Graph gf;
    if (fuse_reduced_axes(*desc, fused)) {
      const syno_desc df = fused.view();
      if (parse_graph(&df, gf, nullptr) == SYNO_OK) plan->conv_like = recognise_conv(gf, plan->conv);
    }
  }
  plan->share_window = !plan->conv_like && recognise_share_window(g, plan->window);
  plan->pure_view = recognise_view(g, plan->view);

  for (int which = 0; which < 3; ++which) {
    Launch& L = plan->launch[which];
    const IndexProgram& P = plan->prog[which];
    L.kernel = KERNEL_GENERIC;
    // Few targets with a long sum each: one workgroup per target, lanes share the sum.
    L.coop = (P.n_free >= 512 && P.n_target < (1 << 18)) ? 1 : 0;
    L.workspace = 0;
    if (policy == 1) continue;
    // Kernel choice.  A per-channel window (one input and one output channel per group) has about one
    // flop per byte: stream it.  A Reduce shared with a weight that also carries its own output
    // iterator is a real contraction: MFMA.  Everything else stays on the index-program kernels.
    if (plan->view.n_red == 0 && view_supports(plan, which)) {   // nothing is summed: a stream whatever else it looks like
      L.kernel = KERNEL_BW_VIEW;
      view_configure(plan, which);
    } else if (bandwidth_supports(plan, which)) {
      L.kernel = KERNEL_BW_DEPTHWISE;
      bandwidth_configure(plan, which);
    } else if (window_supports(plan, which)) {
      L.kernel = KERNEL_BW_WINDOW;
      window_configure(plan, which);
    } else if (mfma_supports(plan, which)) {
      L.kernel = plan->in_dtype == SYNO_BF16 ? KERNEL_MFMA_BF16 : KERNEL_MFMA_F32;
      mfma_configure(plan, which);
    } else if (which == SYNO_BWD_WEIGHT && mfma_dw_supports(plan)) {
      L.kernel = plan->in_dtype == SYNO_BF16 ? KERNEL_MFMA_BF16 : KERNEL_MFMA_F32;
      mfma_dw_configure(plan);
    } else if (view_supports(plan, which)) {       // a few sum points per output and separable offsets: gather-and-add
      L.kernel = KERNEL_BW_VIEW;
      view_configure(plan, which);
    }
  }
  // The gradients of a convolution with a Stride below its window (forward runs on the contraction kernel): on the
  // s*s phase planes X[.., s*h'+a, s*w'+b], taken as s*s*C channels, the window moves with stride 1 - tap kh reads
  // phase (kh-p) mod s at row offset floor((kh-p)/s) - so dW is the weight gradient, and dX the forward contraction,
  // of a stride-1 convolution between the upstream gradient and the phase planes, with a space-to-depth view before
  // or after it.  Only the taps that exist are kept (dW) or non-zero (dX): the stride-1 window has more.
  if (policy != 1 && plan->conv_like && plan->conv.sh > 1 &&
      (plan->launch[SYNO_FWD].kernel == KERNEL_MFMA_F32 || plan->launch[SYNO_FWD].kernel == KERNEL_MFMA_BF16)) {
    const ConvLike& c = plan->conv;
    const int s = c.sh;
    auto floor_div = [](int a, int b) { return (a >= 0 ? a : a - b + 1) / b; };
    const int dmin = floor_div(-c.ph, s), dmax = floor_div(c.KH - 1 - c.ph, s);
    const bool fits = c.G == 1 && c.sw == s && c.KH == c.KW && c.ph == c.pw && !c.h_wrap && !c.w_wrap &&
                      c.Hi == s * c.Ho && c.Wi == s * c.Wo && dmin >= -1 && dmax <= 1 && (int64_t)c.Cg * s * s < (1 << 20);
    if (fits) {
      const int window = (dmin == 0 && dmax == 0) ? 1 : 3;
      // a window that only ever reads phase (0, 0) (1x1 without pad): the other phases do not take part, the view is
      // the sub-sampling itself and its scatter leaves the unread pixels of dX zero
      const int ps = (window == 1 && c.KH == 1 && c.ph == 0) ? 1 : s;
      // out[n,c,a,b,h',w'] = X[n, c, s*h'+a, s*w'+b] (times a one-element weight), element type t on both sides;
      // ps = 1: out[n,c,h',w'] = X[n, c, s*h', s*w']
      auto view_plan = [&](syno_dtype t) -> syno_plan* {
        syno_desc d{};
        syno_prim pr[2] = {};
        const syno_dim dims6[6] = {{"n", c.N}, {"c", c.Cg}, {"a", s}, {"b", s}, {"h", c.Ho}, {"w", c.Wo}};
        const syno_dim dims4[4] = {{"n", c.N}, {"c", c.Cg}, {"h", c.Ho}, {"w", c.Wo}};
        const int32_t xin6[4] = {0, 1, 6, 7}, xin4[4] = {0, 1, 4, 5};
        if (ps > 1) {
          for (int k = 0; k < 2; ++k) {
            pr[k].kind = SYNO_SPLIT; pr[k].in[0] = 4 + k; pr[k].in[1] = 2 + k; pr[k].out[0] = 6 + k; pr[k].out[1] = -1;
            pr[k].shift_by = -1;
          }
          d.n_out = 6; d.out_dims = dims6; d.input_coords = xin6;
        } else {
          for (int k = 0; k < 2; ++k) {
            pr[k].kind = SYNO_STRIDE; pr[k].in[0] = 2 + k; pr[k].in[1] = -1; pr[k].out[0] = 4 + k; pr[k].out[1] = -1;
            pr[k].param = s; pr[k].shift_by = -1;
          }
          d.n_out = 4; d.out_dims = dims4; d.input_coords = xin4;
        }
        d.n_prim = 2; d.prims = pr; d.n_in = 4; d.n_w = 0;
        d.weight_coords = nullptr; d.in_dtype = t; d.out_dtype = t;
        syno_plan* ip = new syno_plan();
        if (build_plan(&d, ip, nullptr) != SYNO_OK) { delete ip; return nullptr; }
        return ip;
      };
      // the stride-1 convolution [N, cin, Ho, Wo] -> [N, cout, Ho, Wo] with a window x window kernel [cout, cin, ., .]
      auto conv_plan = [&](int64_t cin, int64_t cout, syno_dtype out_t) -> syno_plan* {
        const syno_dim dims[4] = {{"n", c.N}, {"co", cout}, {"h", c.Ho}, {"w", c.Wo}};
        syno_prim pr[8] = {};
        auto set = [&](int k, syno_prim_kind kind, int i0, int i1, int o0, int o1, int64_t param) {
          pr[k].kind = kind; pr[k].in[0] = i0; pr[k].in[1] = i1; pr[k].out[0] = o0; pr[k].out[1] = o1; pr[k].param = param;
          pr[k].shift_by = -1;
        };
        set(0, SYNO_REDUCE, -1, -1, 4, -1, cin);    set(1, SYNO_SHARE, 4, -1, 5, 6, 0);
        set(2, SYNO_REDUCE, -1, -1, 7, -1, window); set(3, SYNO_SHARE, 7, -1, 8, 9, 0);
        set(4, SYNO_REDUCE, -1, -1, 10, -1, window); set(5, SYNO_SHARE, 10, -1, 11, 12, 0);
        set(6, SYNO_UNFOLD, 2, 8, 13, -1, 0);       set(7, SYNO_UNFOLD, 3, 11, 14, -1, 0);
        const int32_t xin[4] = {0, 5, 13, 14}, win[4] = {1, 6, 9, 12};
        syno_desc d{};
        d.n_out = 4; d.out_dims = dims; d.n_prim = 8; d.prims = pr; d.n_in = 4; d.input_coords = xin; d.n_w = 4;
        d.weight_coords = win; d.in_dtype = desc->in_dtype; d.out_dtype = out_t;
        syno_plan* ip = new syno_plan();
        if (build_plan(&d, ip, nullptr) != SYNO_OK) { delete ip; return nullptr; }
        return ip;
      };
      auto is_mfma = [](const Launch& L) { return L.kernel == KERNEL_MFMA_F32 || L.kernel == KERNEL_MFMA_BF16; };
      auto round_up = [](size_t n) { return (n + 255) & ~(size_t)255; };
      const int64_t CP = (int64_t)c.Cg * ps * ps;
      const int64_t plane_elems = (int64_t)c.N * CP * c.Ho * c.Wo;      // elements of the view's result
      const size_t esz = desc->in_dtype == SYNO_BF16 ? 2 : 4, osz = desc->out_dtype == SYNO_BF16 ? 2 : 4;
      // backward-weight: space-to-depth of X, weight gradient of the stride-1 convolution, the existing taps picked out
      {
        syno_plan* v = view_plan(desc->in_dtype);
        syno_plan* cw = conv_plan(CP, c.Og, SYNO_F32);
        if (v && cw && v->launch[SYNO_FWD].kernel == KERNEL_BW_VIEW && is_mfma(cw->launch[SYNO_BWD_WEIGHT])) {
          plan->phase_view_x = v; plan->phase_conv_dw = cw; plan->phase_window = window; plan->phase_s = ps;
          Launch& L = plan->launch[SYNO_BWD_WEIGHT];
          L.kernel = KERNEL_MFMA_PHASES;
          L.workspace = round_up((size_t)plane_elems * esz) + round_up((size_t)c.Og * CP * window * window * 4) +
                        cw->launch[SYNO_BWD_WEIGHT].workspace;
        } else {
          delete v; delete cw;
        }
      }
      // backward-data: the weights spread over the phases, the forward contraction from the upstream gradient to the
      // phase planes of dX, depth-to-space (the view's scatter)
      {
        syno_plan* v = view_plan(desc->out_dtype);
        syno_plan* cx = conv_plan(c.Og, CP, desc->out_dtype);
        if (v && cx && v->launch[SYNO_BWD_DATA].kernel == KERNEL_BW_VIEW && is_mfma(cx->launch[SYNO_FWD])) {
          plan->phase_view_dx = v; plan->phase_conv_dx = cx; plan->phase_window = window; plan->phase_s = ps;
          Launch& L = plan->launch[SYNO_BWD_DATA];
          L.kernel = KERNEL_MFMA_PHASES;
          L.workspace = round_up((size_t)CP * c.Og * window * window * esz) + round_up((size_t)plane_elems * osz) +
                        cx->launch[SYNO_FWD].workspace + v->launch[SYNO_BWD_DATA].workspace;
        } else {
          delete v; delete cx;
        }
      }
    }
  }
  // A matrix product is a 1x1 convolution with the operands' roles exchanged: W[k,j] is an "image" with k as
  // channels and the contiguous j as pixels, X[i,k] the weight of output channel i, and out[i,j] is laid out
  // channel-major like a convolution result.  Its gradients exchange roles too: dX is that convolution's
  // weight gradient, dW its input gradient (both need an fp32 result type).
  int64_t M = 0, K = 0, N = 0;
  if (policy != 1 && !plan->conv_like && recognise_matmul(g, M, K, N)) {
    // the 1x1 convolution of the product [rows x red] * [red x cols] (nullptr: cols cannot be folded into image rows)
    auto conv_of_product = [&](int64_t rows, int64_t red, int64_t cols) -> syno_plan* {
      const int64_t width = fold_width(cols);
      if (width <= 0) return nullptr;
      const syno_dim dims[4] = {{"n", 1}, {"i", rows}, {"jr", cols / width}, {"jc", width}};
      syno_prim pr[2] = {};
      pr[0].kind = SYNO_REDUCE; pr[0].in[0] = pr[0].in[1] = -1; pr[0].out[0] = 4; pr[0].out[1] = -1; pr[0].param = red;
      pr[0].shift_by = -1;
      pr[1].kind = SYNO_SHARE; pr[1].in[0] = 4; pr[1].in[1] = -1; pr[1].out[0] = 5; pr[1].out[1] = 6;
      pr[1].shift_by = -1;
      const int32_t xin[4] = {0, 5, 2, 3}, win[2] = {1, 6};
      syno_desc inner{};
      inner.n_out = 4; inner.out_dims = dims; inner.n_prim = 2; inner.prims = pr;
      inner.n_in = 4; inner.input_coords = xin; inner.n_w = 2; inner.weight_coords = win;
      inner.in_dtype = desc->in_dtype; inner.out_dtype = desc->out_dtype;
      inner.options = desc->options;
      syno_plan* ip = new syno_plan();
      if (build_plan(&inner, ip, nullptr) != SYNO_OK) { delete ip; return nullptr; }
      return ip;
    };
    auto is_fast = [](const Launch& L) { return L.kernel == KERNEL_MFMA_F32 || L.kernel == KERNEL_MFMA_BF16; };
    if (syno_plan* ip = conv_of_product(M, K, N)) {
      const int map[3] = {SYNO_FWD, SYNO_BWD_WEIGHT, SYNO_BWD_DATA};
      bool any = false;
      for (int which = 0; which < 3; ++which) {
        const Launch& IL = ip->launch[map[which]];
        if (!is_fast(IL) || (which != SYNO_FWD && desc->out_dtype != SYNO_F32)) continue;
        plan->launch[which].kernel = KERNEL_MFMA_TRANSPOSED;
        plan->launch[which].variant = map[which];
        plan->launch[which].workspace = IL.workspace;
        any = true;
      }
      if (any) plan->inner = ip; else delete ip;
    }
    // dX[i,k] = sum_j G[i,j] W[k,j] is the product of G and W^T: with W^T written out (K*N elements, small beside
    // G and dX) it runs on the forward contraction, whose tiles are the best this family has for 1x1 windows
    if (plan->inner && K < (1ll << 31) && N < (1ll << 31)) {
      if (syno_plan* ip = conv_of_product(M, N, K)) {
        const Launch& IL = ip->launch[SYNO_FWD];
        if (is_fast(IL)) {
          Launch& L = plan->launch[SYNO_BWD_DATA];
          L.kernel = KERNEL_MFMA_TRANSPOSED;
          L.variant = kViaTransposedCopy;
          const size_t esz = desc->in_dtype == SYNO_BF16 ? 2 : 4;
          L.workspace = (((size_t)K * N * esz + 255) & ~(size_t)255) + IL.workspace;
          plan->inner_dx = ip;
        } else {
          delete ip;
        }
      }
    }
  }
  return SYNO_OK;
}

}  // namespace syno
