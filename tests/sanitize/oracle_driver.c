/* Runs every entry point of the CPU oracle on small seeded inputs.  Built by tests/test_sanitizers.py together
 * with oracle/acrobat_oracle.c under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle is what every
 * parity claim rests on, so it must not read or write out of bounds either.  Values are checked only for
 * being finite and for the two evaluation orders agreeing bit for bit; the pins proper are in
 * tests/test_oracle_*.py. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_treelstm(int, const int32_t*, const int32_t*, const int32_t*, const int32_t*, int, int, const float*, const float*,
                    const float*, const float*, const float*, double*, double*, int);
int oracle_treelstm_topo(int, const int32_t*, const int32_t*, const int32_t*, const int32_t*, int, int, const float*,
                         const float*, const float*, const float*, const float*, double*, double*);
int oracle_tree_depths(int, const int32_t*, const int32_t*, const int32_t*, int32_t*);
int oracle_tree_schedule(int, const int32_t*, const int32_t*, const int32_t*, int32_t*, int32_t*, int32_t*, int32_t*);
int oracle_mvrnn(int, const int32_t*, const int32_t*, const int32_t*, const int32_t*, int, const float*, const float*,
                 const float*, const float*, double*, double*, int);
int oracle_varlen_lstm(int, const int32_t*, int, int, const float*, const float*, const float*, const float*, double*, double*, int);
int oracle_seq_schedule(int, const int32_t*, int32_t*, int32_t*);
int oracle_birnn(int, const int32_t*, int, int, int, const float*, const float*, const float*, const float*, const float*,
                 const float*, const float*, const float*, const float*, const float*, const float*, double*, double*, double*, int);
int oracle_phase_schedule(int, const int32_t*, const int32_t*, const int32_t*, int32_t*, int32_t*, int32_t*);
int oracle_drnn(int, int, int, int, const float*, const float*, const float*, const float*, const float*, const float*,
                const float*, const float*, const float*, const float*, uint64_t, int, int, double, double, int, int, int32_t*,
                int32_t*, int32_t*, int32_t*, int32_t*, int32_t*, double*, double*, double*, double*);

static uint64_t state = 0x2545F4914F6CDD1Dull;
static uint32_t rnd(void) { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return (uint32_t)(state >> 32); }
static float unif(float s) { return s * ((float)(rnd() % 20001) / 10000.0f - 1.0f); }
static float* randf(size_t n, float s) {
  float* p = (float*)malloc(sizeof(float) * (n ? n : 1));
  for (size_t i = 0; i < n; ++i) p[i] = unif(s);
  return p;
}
static void check_finite(const double* p, size_t n, const char* what) {
  for (size_t i = 0; i < n; ++i)
    if (!isfinite(p[i])) { printf("%s: element %zu is not finite\n", what, i); exit(1); }
}

int main(void) {
  /* a forest: trees of 1..9 leaves, leaves first, internal nodes joined left to right at random */
  enum { MAXN = 400 };
  int32_t tree_off[16] = {0}, left[MAXN], right[MAXN], token[MAXN];
  int n_trees = 0, N = 0;
  for (; n_trees < 12; ++n_trees) {
    const int leaves = 1 + (int)(rnd() % 9), n = 2 * leaves - 1;
    int roots[16], nr = leaves, next = leaves;
    for (int i = 0; i < n; ++i) { left[N + i] = right[N + i] = -1; token[N + i] = (int32_t)(rnd() % 20); }
    for (int i = 0; i < leaves; ++i) roots[i] = i;
    while (nr > 1) {
      const int k = (int)(rnd() % (uint32_t)(nr - 1));
      left[N + next] = roots[k]; right[N + next] = roots[k + 1];
      roots[k] = next++;
      for (int i = k + 1; i + 1 < nr; ++i) roots[i] = roots[i + 1];
      --nr;
    }
    N += n;
    tree_off[n_trees + 1] = N;
  }
  const int H = 8, D = 6, V = 20;
  float *emb = randf((size_t)V * D, 1.0f), *Wl = randf((size_t)5 * H * D, 0.4f), *bl = randf(5 * H, 0.2f);
  float *U = randf((size_t)5 * H * 2 * H, 0.3f), *b = randf(5 * H, 0.2f);
  double* h = (double*)malloc(sizeof(double) * N * H), *c = (double*)malloc(sizeof(double) * N * H);
  double* h2 = (double*)malloc(sizeof(double) * N * H), *c2 = (double*)malloc(sizeof(double) * N * H);
  oracle_treelstm(n_trees, tree_off, left, right, token, H, D, emb, Wl, bl, U, b, h, c, 1);
  oracle_treelstm(n_trees, tree_off, left, right, token, H, D, emb, Wl, NULL, U, NULL, h2, c2, 3);
  oracle_treelstm_topo(n_trees, tree_off, left, right, token, H, D, emb, Wl, bl, U, b, h2, c2);
  check_finite(h, (size_t)N * H, "treelstm h");
  if (memcmp(h, h2, sizeof(double) * N * H) || memcmp(c, c2, sizeof(double) * N * H)) { printf("recursive != topological\n"); return 1; }
  int32_t depth[MAXN], level_off[MAXN + 1], level_nodes[MAXN], lrow[MAXN], rrow[MAXN];
  const int levels = oracle_tree_depths(n_trees, tree_off, left, right, depth);
  if (oracle_tree_schedule(n_trees, tree_off, left, right, level_off, level_nodes, lrow, rrow) != levels) { printf("levels differ\n"); return 1; }
  oracle_tree_schedule(n_trees, tree_off, left, right, level_off, level_nodes, NULL, NULL);
  if (level_off[levels] != N) { printf("schedule does not cover the forest\n"); return 1; }
  /* MV-RNN */
  const int d = 4;
  float *vt = randf((size_t)V * d, 1.0f), *mt = randf((size_t)V * d * d, 0.5f), *W = randf((size_t)d * 2 * d, 0.3f), *WM = randf((size_t)d * 2 * d, 0.3f);
  double* vec = (double*)malloc(sizeof(double) * N * d), *mat = (double*)malloc(sizeof(double) * N * d * d);
  oracle_mvrnn(n_trees, tree_off, left, right, token, d, vt, mt, W, WM, vec, mat, 2);
  check_finite(vec, (size_t)N * d, "mvrnn vec");
  check_finite(mat, (size_t)N * d * d, "mvrnn mat");
  /* LSTM and bidirectional RNN over ragged sequences, some empty */
  enum { NS = 9 };
  int32_t len[NS];
  int R = 0;
  for (int s = 0; s < NS; ++s) { len[s] = (int32_t)(rnd() % 7); R += len[s]; }
  len[3] = 0;
  R = 0;
  for (int s = 0; s < NS; ++s) R += len[s];
  float *x = randf((size_t)R * D, 1.0f), *Wx = randf((size_t)4 * H * D, 0.4f), *Wh = randf((size_t)4 * H * H, 0.4f), *b4 = randf(4 * H, 0.2f);
  double* lh = (double*)malloc(sizeof(double) * (R ? R : 1) * H), *lc = (double*)malloc(sizeof(double) * (R ? R : 1) * H);
  oracle_varlen_lstm(NS, len, H, D, x, Wx, Wh, b4, lh, lc, 2);
  oracle_varlen_lstm(NS, len, H, D, x, Wx, Wh, NULL, lh, lc, 1);
  check_finite(lh, (size_t)R * H, "lstm h");
  int32_t soff[16], srows[64];
  if (oracle_seq_schedule(NS, len, soff, srows) > 6) { printf("more steps than the longest sequence\n"); return 1; }
  const int n_out = 3;
  float *C = randf((size_t)n_out * 2 * H, 0.3f), *cb = randf(n_out, 0.2f), *fi = randf(H, 0.5f), *bi = randf(H, 0.5f);
  float *fWx = randf((size_t)H * D, 0.4f), *fWh = randf((size_t)H * H, 0.4f), *bWx = randf((size_t)H * D, 0.4f), *bWh = randf((size_t)H * H, 0.4f);
  double* hf = (double*)malloc(sizeof(double) * (R ? R : 1) * H), *hb = (double*)malloc(sizeof(double) * (R ? R : 1) * H);
  double* y = (double*)malloc(sizeof(double) * (R ? R : 1) * n_out);
  oracle_birnn(NS, len, H, D, n_out, x, fWx, fWh, b4, fi, bWx, bWh, NULL, bi, C, cb, hf, hb, y, 2);
  check_finite(y, (size_t)R * n_out, "birnn y");
  /* phase schedule of a small graph: a chain in phase 0, consumers in phase 1 */
  {
    const int32_t prod_off[6] = {0, 0, 1, 2, 4, 5}, prod[5] = {0, 1, 1, 2, 3}, phase[5] = {0, 0, 0, 1, 1};
    int32_t dep[5], order[5], boff[8];
    const int nb = oracle_phase_schedule(5, prod_off, prod, phase, dep, order, boff);
    if (nb < 1 || boff[nb] != 5) { printf("phase schedule does not cover the graph\n"); return 1; }
  }
  /* tree generation, both decision modes, and a capacity that is too small */
  {
    const int n_inst = 4, nl = 5, no = 8, cap = 600;
    float *x0 = randf((size_t)n_inst * H, 1.0f), *e = randf((size_t)nl * H, 1.0f), *Wa = randf((size_t)H * 2 * H, 0.5f), *Wf = randf((size_t)H * 2 * H, 0.5f);
    float *Wp = randf((size_t)H * 2 * H, 0.5f), *Wo = randf((size_t)no * H, 0.5f), *ba = randf(H, 0.2f), *bo = randf(no, 0.2f);
    int32_t* ti = (int32_t*)malloc(sizeof(int32_t) * 6 * cap);
    double* st = (double*)malloc(sizeof(double) * cap * (3 * H + no));
    for (int mode = 0; mode < 2; ++mode) {
      const int n = oracle_drnn(n_inst, H, nl, no, x0, e, Wa, ba, Wf, NULL, Wp, ba, Wo, bo, 99, 4, 3, 0.7, 0.6, mode, cap, ti, ti + cap,
                                ti + 2 * cap, ti + 3 * cap, ti + 4 * cap, ti + 5 * cap, st, st + (size_t)cap * H, st + (size_t)2 * cap * H,
                                st + (size_t)3 * cap * H);
      if (n < n_inst || n > cap) { printf("tree generation: %d nodes\n", n); return 1; }
      check_finite(st, (size_t)n * H, "drnn a");
    }
    if (oracle_drnn(n_inst, H, nl, no, x0, e, Wa, ba, Wf, NULL, Wp, ba, Wo, bo, 99, 4, 3, 0.7, 0.6, 0, 2, ti, ti + cap, ti + 2 * cap,
                    ti + 3 * cap, ti + 4 * cap, ti + 5 * cap, st, st + (size_t)cap * H, st + (size_t)2 * cap * H, st + (size_t)3 * cap * H) != -1) {
      printf("a capacity of 2 nodes was not refused\n");
      return 1;
    }
    free(x0); free(e); free(Wa); free(Wf); free(Wp); free(Wo); free(ba); free(bo); free(ti); free(st);
  }
  free(emb); free(Wl); free(bl); free(U); free(b); free(h); free(c); free(h2); free(c2);
  free(vt); free(mt); free(W); free(WM); free(vec); free(mat);
  free(x); free(Wx); free(Wh); free(b4); free(lh); free(lc);
  free(C); free(cb); free(fi); free(bi); free(fWx); free(fWh); free(bWx); free(bWh); free(hf); free(hb); free(y);
  printf("oracle under the sanitizers: ok\n");
  return 0;
}
