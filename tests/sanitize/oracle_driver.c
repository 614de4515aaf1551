/* Exerciser of the CPU checker for its sanitizer build (gcc -fsanitize=address,undefined).  Same input file as the
 * planner's driver; every description the checker accepts and that is small enough is evaluated forwards and
 * backwards on deterministic data, and its index map is sampled. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_describe(const int64_t*, int64_t, int64_t*, int64_t*, int64_t*, int64_t*, int64_t*, int64_t*);
int oracle_forward(const int64_t*, int64_t, const double*, const double*, double*);
int oracle_forward_at(const int64_t*, int64_t, const double*, const double*, const int64_t*, int64_t, double*);
int oracle_backward(const int64_t*, int64_t, const double*, const double*, const double*, double*, double*,
                    const int64_t*, int64_t, const int64_t*, int64_t);
int oracle_gather_map(const int64_t*, int64_t, const int64_t*, const int64_t*, int64_t, int32_t*, int32_t*);

int main(int argc, char** argv) {
  if (argc < 2) return 2;
  FILE* f = fopen(argv[1], "r");
  if (!f) return 2;
  long long nw;
  int line = 0, evaluated = 0;
  while (fscanf(f, "%lld", &nw) == 1) {
    ++line;
    int64_t* w = malloc(sizeof(int64_t) * (size_t)(nw + 2));
    for (long long i = 0; i < nw + 2; ++i) { long long v; if (fscanf(f, "%lld", &v) != 1) return 2; w[i] = v; }
    int64_t xr, wr, nr, xs[16], ws[16], rs[64];
    if (oracle_describe(w, nw, &xr, xs, &wr, ws, &nr, rs) == 0) {
      int64_t nx = 1, nwt = 1, no = 1, nred = 1;
      for (int i = 0; i < xr; ++i) nx *= xs[i];
      for (int i = 0; i < wr; ++i) nwt *= ws[i];
      for (int i = 0; i < nr; ++i) nred *= rs[i];
      for (int i = 0; i < (int)w[0]; ++i) no *= w[1 + i];
      if (nx <= 200000 && nwt <= 200000 && no <= 200000 && no * nred <= 4000000) {
        double *X = malloc(sizeof(double) * (size_t)nx), *W = malloc(sizeof(double) * (size_t)nwt);
        double *G = malloc(sizeof(double) * (size_t)no), *O = malloc(sizeof(double) * (size_t)no);
        double *dX = malloc(sizeof(double) * (size_t)nx), *dW = malloc(sizeof(double) * (size_t)nwt);
        for (int64_t i = 0; i < nx; ++i) X[i] = (double)((i * 37) % 11) - 5.0;
        for (int64_t i = 0; i < nwt; ++i) W[i] = (double)((i * 17) % 7) - 3.0;
        for (int64_t i = 0; i < no; ++i) G[i] = (double)((i * 29) % 5) - 2.0;
        if (oracle_forward(w, nw, X, W, O)) return 1;
        if (oracle_backward(w, nw, X, W, G, dX, dW, NULL, 0, NULL, 0)) return 1;
        int64_t of[4] = {0, no - 1, no / 2, no / 3}, rf[4] = {0, nred - 1, nred / 2, 0};
        int32_t xo[4], wo[4];
        double at[4];
        if (oracle_gather_map(w, nw, of, rf, 4, xo, wo)) return 1;
        if (oracle_forward_at(w, nw, X, W, of, 4, at)) return 1;
        for (int i = 0; i < 4; ++i) if (at[i] != O[of[i]]) { fprintf(stderr, "line %d: forward_at differs\n", line); return 1; }
        free(X); free(W); free(G); free(O); free(dX); free(dW);
        ++evaluated;
      }
    }
    free(w);
  }
  fclose(f);
  printf("descriptors %d evaluated %d\n", line, evaluated);
  return 0;
}
