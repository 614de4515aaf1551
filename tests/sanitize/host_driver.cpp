// Host-side exerciser of the GPU library's planner for the sanitizer build (AddressSanitizer + UndefinedBehavior-
// Sanitizer on host code only; no kernel is launched and no GPU is needed).  Reads operator descriptions, one per
// line, as integers:  n_words  words...  in_dtype  out_dtype   with the words laid out as
//   n_out, size[n_out], n_prim, n_prim x {kind, in0, in1, out0, out1, param, shift_by, shift_coef},
//   n_in, coord[n_in], n_w, coord[n_w]
// builds plans under several option sets, evaluates the lowered index maps of all three passes on the host at
// pseudo-random points, and runs the materialised-reduction pass.  Exit status 0 unless the library misbehaves
// (the sanitizers abort the process on a finding).
#include <cinttypes>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "syno.h"

static uint64_t lcg(uint64_t& s) { s = s * 6364136223846793005ull + 1442695040888963407ull; return s >> 33; }

int main(int argc, char** argv) {
  if (argc < 2) return 2;
  FILE* f = fopen(argv[1], "r");
  if (!f) return 2;
  long long nw;
  int line = 0, planned = 0, rejected = 0;
  while (fscanf(f, "%lld", &nw) == 1) {
    ++line;
    std::vector<long long> w((size_t)nw + 2);
    for (auto& v : w) if (fscanf(f, "%lld", &v) != 1) return 2;
    size_t p = 0;
    const int n_out = (int)w[p++];
    std::vector<syno_dim> dims((size_t)n_out);
    for (auto& d : dims) { d.name = nullptr; d.size = w[p++]; }
    const int n_prim = (int)w[p++];
    std::vector<syno_prim> prims((size_t)n_prim);
    for (auto& q : prims) {
      q.kind = (syno_prim_kind)w[p++];
      q.in[0] = (int32_t)w[p++]; q.in[1] = (int32_t)w[p++];
      q.out[0] = (int32_t)w[p++]; q.out[1] = (int32_t)w[p++];
      q.param = w[p++]; q.shift_by = (int32_t)w[p++]; q.shift_coef = w[p++];
    }
    const int n_in = (int)w[p++];
    std::vector<int32_t> xin((size_t)n_in);
    for (auto& c : xin) c = (int32_t)w[p++];
    const int n_w = (int)w[p++];
    std::vector<int32_t> win((size_t)n_w);
    for (auto& c : win) c = (int32_t)w[p++];
    syno_desc d{};
    d.n_out = n_out; d.out_dims = dims.data(); d.n_prim = n_prim; d.prims = prims.data();
    d.n_in = n_in; d.input_coords = xin.data(); d.n_w = n_w; d.weight_coords = win.data();
    d.in_dtype = (syno_dtype)w[p++]; d.out_dtype = (syno_dtype)w[p++];

    // option sets: the planner's own choice, the generic kernels, named tile variants, other split targets
    std::vector<syno_plan_options> opts(1);
    opts.push_back(syno_plan_options{1, 0, 0, 0, 0, 0});
    for (int v = -1; v <= 14; ++v)
      for (int rows : {1, 2, 4, 7}) opts.push_back(syno_plan_options{0, v, rows, v & 1, 0, 0});
    opts.push_back(syno_plan_options{0, 0, 0, 0, 1, 3});
    opts.push_back(syno_plan_options{0, 0, 0, 0, 4096, 100000});
    for (size_t oi = 0; oi < opts.size(); ++oi) {
      d.options = oi ? &opts[oi] : nullptr;
      syno_plan* plan = nullptr;
      const syno_status st = syno_plan_create(&d, &plan);
      if (st != SYNO_OK) { if (!oi) ++rejected; continue; }
      if (!oi) ++planned;
      int32_t xr, wr, orr;
      int64_t xs[8], ws[8], os[8];
      if (syno_plan_shapes(plan, &xr, xs, &wr, ws, &orr, os) != SYNO_OK) return 1;
      int64_t n_t[3] = {1, 1, 1};
      for (int i = 0; i < orr; ++i) n_t[0] *= os[i];
      for (int i = 0; i < xr; ++i) n_t[1] *= xs[i];
      for (int i = 0; i < wr; ++i) n_t[2] *= ws[i];
      char buf[600];
      for (int which = 0; which < 3; ++which) {
        size_t bytes = 0;
        if (syno_plan_workspace_bytes(plan, which, &bytes) != SYNO_OK) return 1;
        if (syno_plan_describe(plan, which, buf, sizeof buf) != SYNO_OK || !syno_plan_kernel(plan, which)) return 1;
        if (oi > 1) continue;        // the index maps do not depend on the tile options
        int64_t n_free = 0;
        if (syno_plan_free_size(plan, which, &n_free) != SYNO_OK) return 1;
        const int n = 512;
        std::vector<int64_t> t(n), q(n);
        std::vector<int32_t> a(n), b(n);
        uint64_t seed = 1234567 + (uint64_t)line * 3 + (uint64_t)which;
        for (int i = 0; i < n; ++i) { t[i] = (int64_t)(lcg(seed) % (uint64_t)n_t[which]); q[i] = (int64_t)(lcg(seed) % (uint64_t)n_free); }
        t[0] = 0; q[0] = 0; t[1] = n_t[which] - 1; q[1] = n_free - 1; t[2] = -1; q[3] = n_free;    // edges and out of range
        if (syno_debug_gather_host(plan, which, t.data(), q.data(), n, a.data(), b.data()) != SYNO_OK) return 1;
        const int64_t lim_a = which == 0 ? n_t[1] : n_t[0], lim_b = which == 2 ? n_t[1] : n_t[2];
        for (int i = 0; i < n; ++i)
          if (a[i] < -1 || a[i] >= lim_a || b[i] < -1 || b[i] >= lim_b) { fprintf(stderr, "line %d: offset out of range\n", line); return 1; }
      }
      syno_plan_destroy(plan);
    }
    d.options = nullptr;
    syno_chain* chain = nullptr;
    if (syno_chain_create_materialized(&d, &chain) == SYNO_OK) {
      const int ns = syno_chain_stages(chain);
      size_t bytes = 0;
      for (int i = 0; i <= ns; ++i) (void)syno_chain_plan(chain, i);
      if (syno_chain_workspace_bytes(chain, 0, &bytes) != SYNO_OK || syno_chain_workspace_bytes(chain, 1, &bytes) != SYNO_OK) return 1;
      syno_chain_destroy(chain);
    }
  }
  fclose(f);
  printf("descriptors %d planned %d rejected %d\n", line, planned, rejected);
  return 0;
}
