/*
 * CPU oracle for the batched dataflow-graph hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Only the tests, the smoke check and the benchmark's cpu-baseline leg may load
 * this file.  It shares no code with the GPU path and the GPU path never calls it.
 *
 * What it computes.  Auto-batching changes *when* a cell is evaluated, never
 * *what* is evaluated: lazy dataflow-graph construction plus batching of
 * same-depth nodes is semantics preserving (paper section 2.2 "Dynamic
 * Batching", section 4.1 goal G.1).  So the oracle is the plain definition:
 * every input instance is evaluated on its own, node by node, by recursion over
 * its structure, in double precision on the (exactly converted) fp32 inputs.
 * No levels, no gathers, no arena, no blocking, no fusion.
 *
 * The paper prints no cell equations; it names the models (table 3: TreeLSTM,
 * MV-RNN; listing 1: a recurrent cell applied along a list) and cites their
 * source papers.  The cells below are the standard forms of those models:
 *
 *   binary TreeLSTM, gates (i, f_l, f_r, o, u), each with its own weight block:
 *     leaf:      z = W_leaf x + b_leaf,  x = E[token],  children's h and c are the
 *                shared constant zero state (Evaluation, "Overall Performance": the leaf state is a
 *                constant tensor created once)
 *     internal:  z = U [h_l ; h_r] + b   (the input transform only exists at
 *                leaves: it is the hoisted, depth-0 part; appendix "Operator Hoisting")
 *     i=s(z[0:H]) f_l=s(z[H:2H]) f_r=s(z[2H:3H]) o=s(z[3H:4H]) u=tanh(z[4H:5H])
 *     c = i*u + f_l*c_l + f_r*c_r        h = o*tanh(c)       s(t)=1/(1+exp(-t))
 *
 *   MV-RNN (each node carries a vector and a matrix; left child (a,A), right (b,B)):
 *     p = tanh(W [B a ; A b])     P = W_M [A ; B]     (Evaluation, "Overall Performance": the model
 *     multiplies two intermediate activations); a leaf's (a,A) are table rows.
 *
 *   LSTM along a sequence (listing 1/2 structure, appendix "Exploiting Data Reuse" "four gates"):
 *     z = W_x x_t + W_h h_{t-1} + b, gates (i, f, o, u),
 *     c_t = f*c_{t-1} + i*u,  h_t = o*tanh(c_t),  h_{-1} = c_{-1} = 0.
 *
 *   bidirectional RNN with a per-token output layer (listing 1's cell in both directions,
 *   appendix "Exploiting Data Reuse" (code duplication); output operators as in token classification, Evaluation, "Benefits of Optimizations"):
 *     forward:   hf_t = s(Wf_x x_t + bf + Wf_h hf_{t-1}),  hf_{-1} = f_init (a parameter)
 *     backward:  hb_t = s(Wb_x x_t + bb + Wb_h hb_{t+1}),  hb_{len} = b_init (same cell on the
 *                reversed sequence, own parameters)
 *     output:    y_t = relu(c_b + C [hf_t ; hb_t])
 *
 *   schedule: depth of a node = 0 if it consumes nothing produced inside the
 *     graph, else 1 + max depth of its producers (footnote of section 4.1);
 *     nodes run by increasing depth.  Order inside one depth is a convention
 *     (ascending global node id): members of a batch are independent.
 *
 *   program phases (section 4.1, appendix "Combating Eagerness of Depth Scheduling"): operators of a phase are scheduled and
 *     executed before any operator of the next phase, so depth is counted inside a phase: a
 *     node's depth is 0 if it has no producer in its own phase.
 *
 *   doubly recurrent network generating a tree top-down (table 3 names the model and cites its
 *   source; the recurrent unit is listing 1's cell, as for the other recurrent models).  Node i
 *   of an instance, with parent p and previous sibling q:
 *     a_i = s(W_a [a_p ; E[l_p]] + b_a)     ancestral state; the root takes a_p = the instance's
 *                                           input vector and l_p = 0
 *     f_i = s(W_f [f_q ; E[l_q]] + b_f)     fraternal state; a first child (and the root) takes
 *                                           f_q = 0 and l_q = 0
 *     g_i = s(W_p [a_i ; f_i] + b_p)        predictive state
 *     y_i = W_o g_i + b_o                   scores: has children, has a next sibling, labels
 *   Whether i gets children, whether a sibling follows it, and its label l_i are decisions taken
 *   once y_i exists (tensor-dependent control flow, section 4.2).  As in the paper's evaluation
 *   (Evaluation, "Overall Performance") they are emulated pseudo-randomly: a counter-based generator keyed by the
 *   node's position (instance, path of child indices from the root), so the tree an instance
 *   grows does not depend on the order in which nodes are evaluated.  Alternatively they are read
 *   off the scores: children iff y[0] > 0 (and the depth limit allows), a sibling follows iff
 *   y[1] > 0 (and the limit on children allows), label = first index of the largest label score.
 *   The program is the plain recursion: a node, then its children left to right, each with its
 *   whole subtree.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py (hand
 * computed 1- and 3-node trees, closed forms, library LSTM cells, brute force).
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double sigm(double t) { return 1.0 / (1.0 + exp(-t)); }

/* y[r] = bias[r] + sum_k W[r*ld + k] * x[k],  r in [0,rows) */
static void matvec(const float* W, int rows, int cols, int ld, const double* x,
                   const float* bias, double* y) {
  for (int r = 0; r < rows; ++r) {
    double acc = bias ? (double)bias[r] : 0.0;
    const float* w = W + (size_t)r * ld;
    for (int k = 0; k < cols; ++k) acc += (double)w[k] * x[k];
    y[r] = acc;
  }
}

/* ------------------------------------------------------------------------- */
/* TreeLSTM                                                                   */
/* ------------------------------------------------------------------------- */
typedef struct {
  int H, D;
  const int32_t *left, *right, *token; /* global arrays, children tree-local */
  const float *emb, *Wleaf, *bleaf, *U, *b;
  double *h, *c; /* [N,H] */
} tl_model;

/* the cell of one node; its children (if any) must already be evaluated */
static void treelstm_cell(const tl_model* m, int base, int j, double* z, double* in) {
  const int H = m->H, D = m->D;
  const int g = base + j;
  const double *cl = NULL, *cr = NULL;
  if (m->left[g] < 0) {
    const float* x = m->emb + (size_t)m->token[g] * D;
    for (int k = 0; k < D; ++k) in[k] = (double)x[k];
    matvec(m->Wleaf, 5 * H, D, D, in, m->bleaf, z);
  } else {
    const int gl = base + m->left[g], gr = base + m->right[g];
    for (int k = 0; k < H; ++k) in[k] = m->h[(size_t)gl * H + k];
    for (int k = 0; k < H; ++k) in[H + k] = m->h[(size_t)gr * H + k];
    matvec(m->U, 5 * H, 2 * H, 2 * H, in, m->b, z);
    cl = m->c + (size_t)gl * H;
    cr = m->c + (size_t)gr * H;
  }
  for (int q = 0; q < H; ++q) {
    const double i = sigm(z[q]);
    const double fl = sigm(z[H + q]);
    const double fr = sigm(z[2 * H + q]);
    const double o = sigm(z[3 * H + q]);
    const double u = tanh(z[4 * H + q]);
    const double c_l = cl ? cl[q] : 0.0;
    const double c_r = cr ? cr[q] : 0.0;
    const double c = i * u + fl * c_l + fr * c_r;
    m->c[(size_t)g * H + q] = c;
    m->h[(size_t)g * H + q] = o * tanh(c);
  }
}

static void treelstm_rec(const tl_model* m, int base, int j, double* z, double* in) {
  const int g = base + j;
  if (m->left[g] >= 0) {
    treelstm_rec(m, base, m->left[g], z, in);
    treelstm_rec(m, base, m->right[g], z, in);
  }
  treelstm_cell(m, base, j, z, in);
}

/* root of a tree = the one node that is nobody's child; -1 if the tree is empty */
static int find_root(const int32_t* left, const int32_t* right, int base, int n) {
  if (n <= 0) return -1;
  char* is_child = (char*)calloc((size_t)n, 1);
  for (int j = 0; j < n; ++j) {
    if (left[base + j] >= 0) is_child[left[base + j]] = 1;
    if (right[base + j] >= 0) is_child[right[base + j]] = 1;
  }
  int root = -1;
  for (int j = 0; j < n; ++j)
    if (!is_child[j]) { root = j; break; }
  free(is_child);
  return root;
}

typedef struct {
  const tl_model* m;
  const int32_t* tree_off;
  int n_trees, tid, nthreads;
} tl_job;

static void* treelstm_worker(void* p) {
  const tl_job* jb = (const tl_job*)p;
  const tl_model* m = jb->m;
  const int zin = 5 * m->H, kin = (2 * m->H > m->D ? 2 * m->H : m->D);
  double* z = (double*)malloc(sizeof(double) * (size_t)zin);
  double* in = (double*)malloc(sizeof(double) * (size_t)kin);
  for (int t = jb->tid; t < jb->n_trees; t += jb->nthreads) {
    const int base = jb->tree_off[t], n = jb->tree_off[t + 1] - base;
    const int root = find_root(m->left, m->right, base, n);
    if (root >= 0) treelstm_rec(m, base, root, z, in);
  }
  free(z);
  free(in);
  return NULL;
}

/* Recursive per-tree evaluation.  nthreads > 1 only fans whole trees out over
 * host threads (instances are independent); the per-tree code is the same. */
int oracle_treelstm(int n_trees, const int32_t* tree_off, const int32_t* left,
                    const int32_t* right, const int32_t* token, int H, int D,
                    const float* emb, const float* Wleaf, const float* bleaf, const float* U,
                    const float* b, double* h, double* c, int nthreads) {
  tl_model m = {H, D, left, right, token, emb, Wleaf, bleaf, U, b, h, c};
  if (nthreads < 1) nthreads = 1;
  if (nthreads > 256) nthreads = 256;
  tl_job jobs[256];
  pthread_t th[256];
  for (int i = 0; i < nthreads; ++i) {
    jobs[i].m = &m; jobs[i].tree_off = tree_off; jobs[i].n_trees = n_trees;
    jobs[i].tid = i; jobs[i].nthreads = nthreads;
  }
  if (nthreads == 1) { treelstm_worker(&jobs[0]); return 0; }
  for (int i = 0; i < nthreads; ++i) pthread_create(&th[i], NULL, treelstm_worker, &jobs[i]);
  for (int i = 0; i < nthreads; ++i) pthread_join(th[i], NULL);
  return 0;
}

/* ------------------------------------------------------------------------- */
/* schedule oracle: depth by memoised recursion, then (depth, id) order       */
/* ------------------------------------------------------------------------- */
static int depth_rec(const int32_t* left, const int32_t* right, int base, int j, int32_t* depth) {
  const int g = base + j;
  if (depth[g] >= 0) return depth[g];
  int d = 0;
  if (left[g] >= 0) {
    const int dl = depth_rec(left, right, base, left[g], depth);
    const int dr = depth_rec(left, right, base, right[g], depth);
    d = 1 + (dl > dr ? dl : dr);
  }
  depth[g] = d;
  return d;
}

/* depth[N] out; returns the number of levels (max depth + 1), 0 if N == 0 */
int oracle_tree_depths(int n_trees, const int32_t* tree_off, const int32_t* left,
                       const int32_t* right, int32_t* depth) {
  const int N = tree_off[n_trees];
  int maxd = -1;
  for (int g = 0; g < N; ++g) depth[g] = -1;
  for (int t = 0; t < n_trees; ++t) {
    const int base = tree_off[t], n = tree_off[t + 1] - base;
    for (int j = 0; j < n; ++j) {
      const int d = depth_rec(left, right, base, j, depth);
      if (d > maxd) maxd = d;
    }
  }
  return maxd + 1;
}

/* level_off[n_levels+1], level_nodes[N]: nodes by increasing depth, ascending id inside one.
 * lrow/rrow[N] (optional): global child rows of the node at each list position, -1 at leaves */
int oracle_tree_schedule(int n_trees, const int32_t* tree_off, const int32_t* left,
                         const int32_t* right, int32_t* level_off, int32_t* level_nodes,
                         int32_t* lrow, int32_t* rrow) {
  const int N = tree_off[n_trees];
  int32_t* depth = (int32_t*)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
  int32_t* base_of = (int32_t*)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
  const int n_levels = oracle_tree_depths(n_trees, tree_off, left, right, depth);
  for (int t = 0; t < n_trees; ++t)
    for (int g = tree_off[t]; g < tree_off[t + 1]; ++g) base_of[g] = tree_off[t];
  int pos = 0;
  level_off[0] = 0;
  for (int d = 0; d < n_levels; ++d) {
    for (int g = 0; g < N; ++g)
      if (depth[g] == d) {
        level_nodes[pos] = g;
        if (lrow) lrow[pos] = left[g] >= 0 ? base_of[g] + left[g] : -1;
        if (rrow) rrow[pos] = right[g] >= 0 ? base_of[g] + right[g] : -1;
        ++pos;
      }
    level_off[d + 1] = pos;
  }
  free(depth);
  free(base_of);
  return n_levels;
}

/* Same cell, but nodes visited in schedule order instead of by recursion
 * (section 4.1, observation O.1: program order and depth order are both valid
 * dependency orders, so both must give the same values). */
int oracle_treelstm_topo(int n_trees, const int32_t* tree_off, const int32_t* left,
                         const int32_t* right, const int32_t* token, int H, int D,
                         const float* emb, const float* Wleaf, const float* bleaf,
                         const float* U, const float* b, double* h, double* c) {
  tl_model m = {H, D, left, right, token, emb, Wleaf, bleaf, U, b, h, c};
  const int N = tree_off[n_trees];
  if (N == 0) return 0;
  int32_t* level_off = (int32_t*)malloc(sizeof(int32_t) * (size_t)(N + 1));
  int32_t* level_nodes = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
  int32_t* base_of = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
  oracle_tree_schedule(n_trees, tree_off, left, right, level_off, level_nodes, NULL, NULL);
  for (int t = 0; t < n_trees; ++t)
    for (int g = tree_off[t]; g < tree_off[t + 1]; ++g) base_of[g] = tree_off[t];
  const int zin = 5 * H, kin = (2 * H > D ? 2 * H : D);
  double* z = (double*)malloc(sizeof(double) * (size_t)zin);
  double* in = (double*)malloc(sizeof(double) * (size_t)kin);
  for (int p = 0; p < N; ++p) {
    const int g = level_nodes[p];
    treelstm_cell(&m, base_of[g], g - base_of[g], z, in);
  }
  free(z); free(in); free(level_off); free(level_nodes); free(base_of);
  return 0;
}

/* ------------------------------------------------------------------------- */
/* MV-RNN                                                                     */
/* ------------------------------------------------------------------------- */
typedef struct {
  int d;
  const int32_t *left, *right, *token;
  const float *vec_tab, *mat_tab, *W, *WM;
  double *vec, *mat; /* [N,d], [N,d,d] */
} mv_model;

static void mvrnn_rec(const mv_model* m, int base, int j, double* v) {
  const int d = m->d;
  const int g = base + j;
  double* p = m->vec + (size_t)g * d;
  double* P = m->mat + (size_t)g * d * d;
  if (m->left[g] < 0) {
    const float* a = m->vec_tab + (size_t)m->token[g] * d;
    const float* A = m->mat_tab + (size_t)m->token[g] * d * d;
    for (int r = 0; r < d; ++r) p[r] = (double)a[r];
    for (int e = 0; e < d * d; ++e) P[e] = (double)A[e];
    return;
  }
  mvrnn_rec(m, base, m->left[g], v);
  mvrnn_rec(m, base, m->right[g], v);
  const int gl = base + m->left[g], gr = base + m->right[g];
  const double *a = m->vec + (size_t)gl * d, *A = m->mat + (size_t)gl * d * d;
  const double *b = m->vec + (size_t)gr * d, *B = m->mat + (size_t)gr * d * d;
  /* v = [B a ; A b] */
  for (int r = 0; r < d; ++r) {
    double s0 = 0.0, s1 = 0.0;
    for (int k = 0; k < d; ++k) s0 += B[r * d + k] * a[k];
    for (int k = 0; k < d; ++k) s1 += A[r * d + k] * b[k];
    v[r] = s0;
    v[d + r] = s1;
  }
  /* p = tanh(W v) */
  for (int r = 0; r < d; ++r) {
    double s = 0.0;
    for (int k = 0; k < 2 * d; ++k) s += (double)m->W[(size_t)r * 2 * d + k] * v[k];
    p[r] = tanh(s);
  }
  /* P = W_M [A ; B]  ([d x 2d] times the vertical stack [2d x d]) */
  for (int r = 0; r < d; ++r)
    for (int q = 0; q < d; ++q) {
      double s = 0.0;
      for (int k = 0; k < d; ++k) s += (double)m->WM[(size_t)r * 2 * d + k] * A[k * d + q];
      for (int k = 0; k < d; ++k) s += (double)m->WM[(size_t)r * 2 * d + d + k] * B[k * d + q];
      P[r * d + q] = s;
    }
}

typedef struct {
  const mv_model* m;
  const int32_t* tree_off;
  int n_trees, tid, nthreads;
} mv_job;

static void* mvrnn_worker(void* p) {
  const mv_job* jb = (const mv_job*)p;
  double* v = (double*)malloc(sizeof(double) * 2 * (size_t)jb->m->d);
  for (int t = jb->tid; t < jb->n_trees; t += jb->nthreads) {
    const int base = jb->tree_off[t], n = jb->tree_off[t + 1] - base;
    const int root = find_root(jb->m->left, jb->m->right, base, n);
    if (root >= 0) mvrnn_rec(jb->m, base, root, v);
  }
  free(v);
  return NULL;
}

int oracle_mvrnn(int n_trees, const int32_t* tree_off, const int32_t* left, const int32_t* right,
                 const int32_t* token, int d, const float* vec_tab, const float* mat_tab,
                 const float* W, const float* WM, double* vec, double* mat, int nthreads) {
  mv_model m = {d, left, right, token, vec_tab, mat_tab, W, WM, vec, mat};
  if (nthreads < 1) nthreads = 1;
  if (nthreads > 256) nthreads = 256;
  mv_job jobs[256];
  pthread_t th[256];
  for (int i = 0; i < nthreads; ++i) {
    jobs[i].m = &m; jobs[i].tree_off = tree_off; jobs[i].n_trees = n_trees;
    jobs[i].tid = i; jobs[i].nthreads = nthreads;
  }
  if (nthreads == 1) { mvrnn_worker(&jobs[0]); return 0; }
  for (int i = 0; i < nthreads; ++i) pthread_create(&th[i], NULL, mvrnn_worker, &jobs[i]);
  for (int i = 0; i < nthreads; ++i) pthread_join(th[i], NULL);
  return 0;
}

/* ------------------------------------------------------------------------- */
/* variable-length LSTM: every sequence on its own                            */
/* ------------------------------------------------------------------------- */
typedef struct {
  int n_seq, H, D;
  const int32_t* len;
  const float *x, *Wx, *Wh, *b;
  double *h, *c;
  int tid, nthreads;
} ls_job;

static void* lstm_worker(void* p) {
  const ls_job* jb = (const ls_job*)p;
  const int H = jb->H, D = jb->D;
  double* zx = (double*)malloc(sizeof(double) * 4 * (size_t)H);
  double* zh = (double*)malloc(sizeof(double) * 4 * (size_t)H);
  double* xin = (double*)malloc(sizeof(double) * (size_t)D);
  double* hprev = (double*)malloc(sizeof(double) * (size_t)H);
  double* cprev = (double*)malloc(sizeof(double) * (size_t)H);
  size_t row0 = 0;
  for (int s = 0; s < jb->n_seq; ++s) {
    const int T = jb->len[s];
    if (s % jb->nthreads == jb->tid) {
      for (int q = 0; q < H; ++q) hprev[q] = cprev[q] = 0.0;
      for (int t = 0; t < T; ++t) {
        const size_t row = row0 + (size_t)t;
        for (int k = 0; k < D; ++k) xin[k] = (double)jb->x[row * D + k];
        matvec(jb->Wx, 4 * H, D, D, xin, jb->b, zx);
        matvec(jb->Wh, 4 * H, H, H, hprev, NULL, zh);
        for (int q = 0; q < H; ++q) {
          const double i = sigm(zx[q] + zh[q]);
          const double f = sigm(zx[H + q] + zh[H + q]);
          const double o = sigm(zx[2 * H + q] + zh[2 * H + q]);
          const double u = tanh(zx[3 * H + q] + zh[3 * H + q]);
          const double c = f * cprev[q] + i * u;
          jb->c[row * H + q] = c;
          jb->h[row * H + q] = o * tanh(c);
        }
        for (int q = 0; q < H; ++q) {
          hprev[q] = jb->h[row * H + q];
          cprev[q] = jb->c[row * H + q];
        }
      }
    }
    row0 += (size_t)T;
  }
  free(zx); free(zh); free(xin); free(hprev); free(cprev);
  return NULL;
}

int oracle_varlen_lstm(int n_seq, const int32_t* len, int H, int D, const float* x,
                       const float* Wx, const float* Wh, const float* b, double* h, double* c,
                       int nthreads) {
  if (nthreads < 1) nthreads = 1;
  if (nthreads > 256) nthreads = 256;
  ls_job jobs[256];
  pthread_t th[256];
  for (int i = 0; i < nthreads; ++i) {
    ls_job j = {n_seq, H, D, len, x, Wx, Wh, b, h, c, i, nthreads};
    jobs[i] = j;
  }
  if (nthreads == 1) { lstm_worker(&jobs[0]); return 0; }
  for (int i = 0; i < nthreads; ++i) pthread_create(&th[i], NULL, lstm_worker, &jobs[i]);
  for (int i = 0; i < nthreads; ++i) pthread_join(th[i], NULL);
  return 0;
}

/* sequence schedule: level t holds the rows (seq_off[s] + t) of all s with len[s] > t,
 * ascending s.  Returns the number of levels (max len). */
int oracle_seq_schedule(int n_seq, const int32_t* len, int32_t* level_off, int32_t* level_rows) {
  int tmax = 0;
  for (int s = 0; s < n_seq; ++s)
    if (len[s] > tmax) tmax = len[s];
  int pos = 0;
  level_off[0] = 0;
  for (int t = 0; t < tmax; ++t) {
    int row0 = 0;
    for (int s = 0; s < n_seq; ++s) {
      if (len[s] > t) level_rows[pos++] = row0 + t;
      row0 += len[s];
    }
    level_off[t + 1] = pos;
  }
  return tmax;
}

/* ------------------------------------------------------------------------- */
/* bidirectional RNN with per-token output layer                              */
/* ------------------------------------------------------------------------- */
typedef struct {
  int n_seq, H, D, n_out;
  const int32_t* len;
  const float *x, *fWx, *fWh, *fb, *finit, *bWx, *bWh, *bb, *binit, *C, *cb;
  double *hf, *hb, *y;
  int tid, nthreads;
} bi_job;

/* one direction of one sequence: rows row0 .. row0+T-1, visited in the order given by `step` */
static void rnn_chain(const bi_job* jb, size_t row0, int T, int backward, const float* Wx,
                      const float* Wh, const float* b, const float* init, double* hout,
                      double* zx, double* zh, double* xin, double* hprev) {
  const int H = jb->H, D = jb->D;
  for (int q = 0; q < H; ++q) hprev[q] = (double)init[q];
  for (int i = 0; i < T; ++i) {
    const int t = backward ? T - 1 - i : i;
    const size_t row = row0 + (size_t)t;
    for (int k = 0; k < D; ++k) xin[k] = (double)jb->x[row * D + k];
    matvec(Wx, H, D, D, xin, b, zx);
    matvec(Wh, H, H, H, hprev, NULL, zh);
    for (int q = 0; q < H; ++q) hout[row * H + q] = sigm(zx[q] + zh[q]);
    for (int q = 0; q < H; ++q) hprev[q] = hout[row * H + q];
  }
}

static void* birnn_worker(void* p) {
  const bi_job* jb = (const bi_job*)p;
  const int H = jb->H, D = jb->D;
  double* zx = (double*)malloc(sizeof(double) * (size_t)H);
  double* zh = (double*)malloc(sizeof(double) * (size_t)H);
  double* xin = (double*)malloc(sizeof(double) * (size_t)D);
  double* hprev = (double*)malloc(sizeof(double) * (size_t)H);
  double* pin = (double*)malloc(sizeof(double) * 2 * (size_t)H);
  double* yo = (double*)malloc(sizeof(double) * (size_t)jb->n_out);
  size_t row0 = 0;
  for (int s = 0; s < jb->n_seq; ++s) {
    const int T = jb->len[s];
    if (s % jb->nthreads == jb->tid) {
      rnn_chain(jb, row0, T, 0, jb->fWx, jb->fWh, jb->fb, jb->finit, jb->hf, zx, zh, xin, hprev);
      rnn_chain(jb, row0, T, 1, jb->bWx, jb->bWh, jb->bb, jb->binit, jb->hb, zx, zh, xin, hprev);
      for (int t = 0; t < T; ++t) {
        const size_t row = row0 + (size_t)t;
        for (int q = 0; q < H; ++q) pin[q] = jb->hf[row * H + q];
        for (int q = 0; q < H; ++q) pin[H + q] = jb->hb[row * H + q];
        matvec(jb->C, jb->n_out, 2 * H, 2 * H, pin, jb->cb, yo);
        for (int o = 0; o < jb->n_out; ++o) jb->y[row * jb->n_out + o] = yo[o] > 0.0 ? yo[o] : 0.0;
      }
    }
    row0 += (size_t)T;
  }
  free(zx); free(zh); free(xin); free(hprev); free(pin); free(yo);
  return NULL;
}

int oracle_birnn(int n_seq, const int32_t* len, int H, int D, int n_out, const float* x,
                 const float* fWx, const float* fWh, const float* fb, const float* finit,
                 const float* bWx, const float* bWh, const float* bb, const float* binit,
                 const float* C, const float* cb, double* hf, double* hb, double* y, int nthreads) {
  if (nthreads < 1) nthreads = 1;
  if (nthreads > 256) nthreads = 256;
  bi_job jobs[256];
  pthread_t th[256];
  for (int i = 0; i < nthreads; ++i) {
    bi_job j = {n_seq, H, D, n_out, len, x, fWx, fWh, fb, finit, bWx, bWh, bb, binit, C, cb, hf, hb, y, i, nthreads};
    jobs[i] = j;
  }
  if (nthreads == 1) { birnn_worker(&jobs[0]); return 0; }
  for (int i = 0; i < nthreads; ++i) pthread_create(&th[i], NULL, birnn_worker, &jobs[i]);
  for (int i = 0; i < nthreads; ++i) pthread_join(th[i], NULL);
  return 0;
}

/* Generic phase-aware depth schedule of an explicit dataflow graph.  Node n has producers
 * prod[prod_off[n] .. prod_off[n+1]) and phase phase[n] (producers never sit in a later phase).
 * depth[n] = 0 if n has no producer in its own phase, else 1 + the largest such producer's
 * depth.  order[] lists the nodes by (phase, depth, id); batch_off[] marks the batches.
 * Returns the number of batches. */
static int phase_depth(int n, const int32_t* prod_off, const int32_t* prod, const int32_t* phase, int32_t* depth) {
  if (depth[n] >= 0) return depth[n];
  int d = 0;
  for (int e = prod_off[n]; e < prod_off[n + 1]; ++e)
    if (phase[prod[e]] == phase[n]) {
      const int dp = 1 + phase_depth(prod[e], prod_off, prod, phase, depth);
      if (dp > d) d = dp;
    }
  depth[n] = d;
  return d;
}

int oracle_phase_schedule(int n_nodes, const int32_t* prod_off, const int32_t* prod, const int32_t* phase,
                          int32_t* depth, int32_t* order, int32_t* batch_off) {
  int max_phase = 0, max_depth = 0;
  for (int n = 0; n < n_nodes; ++n) depth[n] = -1;
  for (int n = 0; n < n_nodes; ++n) {
    const int d = phase_depth(n, prod_off, prod, phase, depth);
    if (d > max_depth) max_depth = d;
    if (phase[n] > max_phase) max_phase = phase[n];
  }
  int pos = 0, nb = 0;
  batch_off[0] = 0;
  for (int ph = 0; ph <= max_phase; ++ph)
    for (int d = 0; d <= max_depth; ++d) {
      const int before = pos;
      for (int n = 0; n < n_nodes; ++n)
        if (phase[n] == ph && depth[n] == d) order[pos++] = n;
      if (pos > before) batch_off[++nb] = pos;
    }
  return nb;
}

/* ------------------------------------------------------------------------- */
/* doubly recurrent network: top-down tree generation                         */
/* ------------------------------------------------------------------------- */
/* One step of the splitmix64 sequence from state z (its published first outputs for state 0
 * are e220a8397b1dcdaf, 6e789e6aa1b965f4, 06c45d188009454f). */
uint64_t oracle_mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

/* Position keys: root of instance s, k-th child of the node with key `parent`. */
uint64_t oracle_drnn_root_key(uint64_t seed, int inst) { return oracle_mix64(seed ^ oracle_mix64((uint64_t)inst)); }
uint64_t oracle_drnn_child_key(uint64_t parent, int k) { return oracle_mix64(parent + (uint64_t)k + 1u); }

static double unit_interval(uint64_t bits) { return (double)(bits >> 11) * (1.0 / 9007199254740992.0); }

/* The emulated decisions of the node at `key`: depth counts from 0 at the root, k is its index
 * among its siblings.  out = {has_child, has_sibling, label}. */
void oracle_drnn_decide(uint64_t key, int depth, int k, int is_root, int max_depth, int max_children,
                        double p_child, double p_sibling, int n_labels, int32_t* out) {
  out[0] = depth + 1 < max_depth && unit_interval(oracle_mix64(key ^ 1u)) < p_child;
  out[1] = !is_root && k + 1 < max_children && unit_interval(oracle_mix64(key ^ 2u)) < p_sibling;
  out[2] = (int32_t)(oracle_mix64(key ^ 3u) % (uint64_t)n_labels);
}

/* The same decisions read off a node's scores y[0 .. n_out). */
void oracle_drnn_decide_from_scores(const double* y, int depth, int k, int is_root, int max_depth, int max_children,
                                    int n_labels, int n_out, int32_t* out) {
  out[0] = depth + 1 < max_depth && y[0] > 0.0;
  out[1] = !is_root && k + 1 < max_children && y[1] > 0.0;
  const int n = n_labels < n_out - 2 ? n_labels : n_out - 2;
  int best = 0;
  for (int l = 1; l < n; ++l)
    if (y[2 + l] > y[2 + best]) best = l;
  out[2] = best;
}

typedef struct {
  int H, n_labels, n_out, max_depth, max_children, cap, from_scores;
  double p_child, p_sibling;
  const float *emb, *Wa, *ba, *Wf, *bf, *Wp, *bp, *Wo, *bo;
  int32_t *inst, *parent, *prev, *sib_index, *depth, *label;
  double *a, *f, *g, *y;
  int n; /* nodes so far */
  double *in, *z;
} dr_model;

/* evaluates one node (parent / prev: node ids or -1) and returns its id, or -1 when out of room */
static int drnn_node(dr_model* m, int inst, int parent, int prev, int k, int depth, const float* x0) {
  if (m->n >= m->cap) return -1;
  const int H = m->H, i = m->n++;
  m->inst[i] = inst; m->parent[i] = parent; m->prev[i] = prev; m->sib_index[i] = k; m->depth[i] = depth;
  double* in = m->in;
  double* z = m->z;
  /* ancestral */
  for (int q = 0; q < H; ++q) in[q] = parent >= 0 ? m->a[(size_t)parent * H + q] : (double)x0[q];
  const float* e = m->emb + (size_t)(parent >= 0 ? m->label[parent] : 0) * H;
  for (int q = 0; q < H; ++q) in[H + q] = (double)e[q];
  matvec(m->Wa, H, 2 * H, 2 * H, in, m->ba, z);
  for (int q = 0; q < H; ++q) m->a[(size_t)i * H + q] = sigm(z[q]);
  /* fraternal */
  for (int q = 0; q < H; ++q) in[q] = prev >= 0 ? m->f[(size_t)prev * H + q] : 0.0;
  e = m->emb + (size_t)(prev >= 0 ? m->label[prev] : 0) * H;
  for (int q = 0; q < H; ++q) in[H + q] = (double)e[q];
  matvec(m->Wf, H, 2 * H, 2 * H, in, m->bf, z);
  for (int q = 0; q < H; ++q) m->f[(size_t)i * H + q] = sigm(z[q]);
  /* predictive state and scores */
  for (int q = 0; q < H; ++q) in[q] = m->a[(size_t)i * H + q];
  for (int q = 0; q < H; ++q) in[H + q] = m->f[(size_t)i * H + q];
  matvec(m->Wp, H, 2 * H, 2 * H, in, m->bp, z);
  for (int q = 0; q < H; ++q) m->g[(size_t)i * H + q] = sigm(z[q]);
  for (int q = 0; q < H; ++q) in[q] = m->g[(size_t)i * H + q];
  matvec(m->Wo, m->n_out, H, H, in, m->bo, m->y + (size_t)i * m->n_out);
  return i;
}

/* the children of `parent` (key pkey, depth pdepth), left to right, each followed by its subtree */
static int drnn_children(dr_model* m, int inst, int parent, uint64_t pkey, int pdepth) {
  int prev = -1;
  for (int k = 0;; ++k) {
    const uint64_t key = oracle_drnn_child_key(pkey, k);
    const int i = drnn_node(m, inst, parent, prev, k, pdepth + 1, NULL);
    if (i < 0) return -1;
    int32_t d[3];
    if (m->from_scores)
      oracle_drnn_decide_from_scores(m->y + (size_t)i * m->n_out, pdepth + 1, k, 0, m->max_depth, m->max_children, m->n_labels, m->n_out, d);
    else
      oracle_drnn_decide(key, pdepth + 1, k, 0, m->max_depth, m->max_children, m->p_child, m->p_sibling, m->n_labels, d);
    m->label[i] = d[2];
    if (d[0] && drnn_children(m, inst, i, key, pdepth + 1) < 0) return -1;
    if (!d[1]) return 0;
    prev = i;
  }
}

/* Generates one tree per instance from x0 [n_inst, H].  Nodes are numbered in the order the
 * recursion visits them (instance by instance, pre-order).  Arrays hold `cap` nodes; returns the
 * number of nodes, or -1 if they do not fit. */
int oracle_drnn(int n_inst, int H, int n_labels, int n_out, const float* x0, const float* emb,
                const float* Wa, const float* ba, const float* Wf, const float* bf, const float* Wp,
                const float* bp, const float* Wo, const float* bo, uint64_t seed, int max_depth,
                int max_children, double p_child, double p_sibling, int from_scores, int cap, int32_t* inst,
                int32_t* parent, int32_t* prev, int32_t* sib_index, int32_t* depth, int32_t* label,
                double* a, double* f, double* g, double* y) {
  dr_model m = {H, n_labels, n_out, max_depth, max_children, cap, from_scores, p_child, p_sibling, emb, Wa, ba, Wf, bf, Wp, bp,
                Wo, bo, inst, parent, prev, sib_index, depth, label, a, f, g, y, 0, NULL, NULL};
  m.in = (double*)malloc(sizeof(double) * 2 * (size_t)H);
  m.z = (double*)malloc(sizeof(double) * (size_t)(H > n_out ? H : n_out));
  int rc = 0;
  for (int s = 0; s < n_inst && rc == 0; ++s) {
    const uint64_t key = oracle_drnn_root_key(seed, s);
    const int i = drnn_node(&m, s, -1, -1, 0, 0, x0 + (size_t)s * H);
    if (i < 0) { rc = -1; break; }
    int32_t d[3];
    if (from_scores) oracle_drnn_decide_from_scores(y + (size_t)i * n_out, 0, 0, 1, max_depth, max_children, n_labels, n_out, d);
    else oracle_drnn_decide(key, 0, 0, 1, max_depth, max_children, p_child, p_sibling, n_labels, d);
    label[i] = d[2];
    if (d[0]) rc = drnn_children(&m, s, i, key, 0);
  }
  free(m.in); free(m.z);
  return rc < 0 ? -1 : m.n;
}
