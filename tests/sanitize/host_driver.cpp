// Exercises the product's host-side code (level schedulers, dataflow-graph runtime, the tree-generation
// program in its sequential mode) on seeded random and malformed inputs.  Built by tests/test_sanitizers.py
// with AddressSanitizer and UndefinedBehaviorSanitizer: the point is that nothing reads or writes out of
// bounds, overflows or uses freed memory, also on the error paths.  No GPU code is involved.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "dfg_runtime.h"
#include "scheduler.h"
#include "tdc_runtime.h"

using namespace acrobat;

namespace {

uint64_t rng_state = 0x9E3779B97F4A7C15ull;
uint32_t rnd() {
  rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
  return (uint32_t)(rng_state >> 32);
}
int rnd_in(int lo, int hi) { return lo + (int)(rnd() % (uint32_t)(hi - lo + 1)); }

#define CHECK(cond)                                                            \
  do {                                                                         \
    if (!(cond)) { std::printf("CHECK failed: %s (line %d)\n", #cond, __LINE__); std::exit(1); } \
  } while (0)

struct Forest {
  std::vector<int32_t> tree_off{0}, left, right, token;
  acrobat_trees view() const { return {(int32_t)tree_off.size() - 1, tree_off.data(), left.data(), right.data(), token.data()}; }
};

// random binary tree over `leaves` leaves: leaves first, internal nodes in post order (root last)
void add_tree(Forest& f, int leaves, int vocab) {
  const int n = 2 * leaves - 1;
  std::vector<int32_t> l(n, -1), r(n, -1);
  int next = leaves;
  struct Span { int lo, hi; };
  // build by repeatedly joining two adjacent subtrees (roots listed left to right)
  std::vector<int> roots(leaves);
  for (int i = 0; i < leaves; ++i) roots[i] = i;
  while (roots.size() > 1) {
    const int k = rnd_in(0, (int)roots.size() - 2);
    l[next] = roots[k]; r[next] = roots[k + 1];
    roots[k] = next++;
    roots.erase(roots.begin() + k + 1);
  }
  // optional random relabelling, so that the scheduler's general path runs too
  std::vector<int> perm(n);
  for (int i = 0; i < n; ++i) perm[i] = i;
  if (rnd() & 1)
    for (int i = n - 1; i > 0; --i) std::swap(perm[i], perm[rnd_in(0, i)]);
  std::vector<int32_t> L(n), R(n), T(n);
  for (int i = 0; i < n; ++i) {
    L[perm[i]] = l[i] < 0 ? -1 : perm[l[i]];
    R[perm[i]] = r[i] < 0 ? -1 : perm[r[i]];
    T[perm[i]] = rnd_in(0, vocab - 1);
  }
  f.left.insert(f.left.end(), L.begin(), L.end());
  f.right.insert(f.right.end(), R.begin(), R.end());
  f.token.insert(f.token.end(), T.begin(), T.end());
  f.tree_off.push_back(f.tree_off.back() + n);
}

int depth_of(const Forest& f, int base, int j) {
  if (f.left[base + j] < 0) return 0;
  const int a = depth_of(f, base, f.left[base + j]), b = depth_of(f, base, f.right[base + j]);
  return 1 + (a > b ? a : b);
}

void check_tree_schedule(const Forest& f, const TreeSchedule& s) {
  const int N = f.tree_off.back();
  CHECK(s.n_nodes == N);
  CHECK((int)s.level_off.size() == s.n_levels + 1 && s.level_off.back() == N);
  std::vector<int> seen(N, 0), tree_of(N, 0);
  for (size_t t = 0; t + 1 < f.tree_off.size(); ++t)
    for (int g = f.tree_off[t]; g < f.tree_off[t + 1]; ++g) tree_of[g] = (int)t;
  for (int lv = 0; lv < s.n_levels; ++lv)
    for (int p = s.level_off[lv]; p < s.level_off[lv + 1]; ++p) {
      const int g = s.level_nodes[p], base = f.tree_off[tree_of[g]];
      CHECK(g >= 0 && g < N && !seen[g]);
      seen[g] = 1;
      CHECK(depth_of(f, base, g - base) == lv);
      if (p > s.level_off[lv]) CHECK(s.level_nodes[p - 1] < g);
      CHECK(s.lrow[p] == (f.left[g] < 0 ? -1 : base + f.left[g]));
      CHECK(s.rrow[p] == (f.right[g] < 0 ? -1 : base + f.right[g]));
    }
}

}  // namespace

int main() {
  std::string err;
  TreeScheduler reuse;
  TreeSchedule kept;
  std::vector<int32_t> toks;
  for (int round = 0; round < 60; ++round) {
    Forest f;
    const int n_trees = rnd_in(0, 12);
    for (int t = 0; t < n_trees; ++t) {
      if (rnd() % 7 == 0) { f.tree_off.push_back(f.tree_off.back()); continue; }  // an empty tree
      add_tree(f, rnd_in(1, 40), 50);
    }
    const acrobat_trees v = f.view();
    TreeSchedule s;
    CHECK(schedule_trees(v, 50, s, err) == ACROBAT_OK);
    check_tree_schedule(f, s);
    CHECK(reuse.begin(v, 50, kept, &toks, err) == ACROBAT_OK);  // buffers reused across rounds of different sizes
    reuse.finish(v, kept);
    check_tree_schedule(f, kept);
    CHECK(kept.level_nodes == s.level_nodes && kept.lrow == s.lrow && kept.rrow == s.rrow);
    CHECK(s.n_levels == 0 || (int)toks.size() == s.level_off[1]);
    for (size_t p = 0; p < toks.size(); ++p) CHECK(toks[p] == f.token[s.level_nodes[p]]);
    // the unbatched TreeLSTM program through invoke(): its buckets are the same levels
    {
      Dfg g;
      acrobat_op_desc leaf{}, internal{};
      leaf.epilogue = ACROBAT_EPI_TREE_LEAF; leaf.H = 32; leaf.nseg = 1; leaf.kseg = 32; leaf.ld0 = 32; leaf.ldw = 32;
      leaf.src0_rows = 50; leaf.out_rows = s.n_nodes > 0 ? s.n_nodes : 1;
      internal = leaf;
      internal.epilogue = ACROBAT_EPI_TREE_INTERNAL; internal.nseg = 2; internal.ld1 = 32; internal.ldw = 64;
      internal.src0_rows = internal.src1_rows = internal.out_rows;
      static float dummy[1];
      leaf.src0 = leaf.W = internal.src0 = internal.src1 = internal.W = internal.cprev_src = dummy;
      leaf.h = leaf.c = internal.h = internal.c = dummy;
      int32_t op_leaf = -1, op_int = -1;
      CHECK(g.register_op(leaf, &op_leaf, err) == ACROBAT_OK);
      CHECK(g.register_op(internal, &op_int, err) == ACROBAT_OK);
      { const int rcb = dfg_build_treelstm(g, v, 50, op_leaf, op_int, err); if (rcb != ACROBAT_OK) std::printf("build: %d %s (nodes %d)\n", rcb, err.c_str(), s.n_nodes); CHECK(rcb == ACROBAT_OK); }
      DfgBuckets b;
      g.bucket(b);
      CHECK((int)b.order.size() == s.n_nodes);
      CHECK((int)b.op.size() == s.n_levels);
      for (int lv = 0; lv < s.n_levels; ++lv) CHECK(b.off[lv + 1] - b.off[lv] == s.level_off[lv + 1] - s.level_off[lv]);
    }
    // malformed variants of the same forest: every one must be refused, none may crash
    if (!f.left.empty()) {
      for (int k = 0; k < 12; ++k) {
        Forest m = f;
        const int g = rnd_in(0, (int)m.left.size() - 1);
        switch (k % 6) {
          case 0: m.left[g] = rnd_in(-5, 1000); break;
          case 1: m.right[g] = m.left[g]; break;
          case 2: m.token[g] = rnd() & 1 ? -1 : 50; break;
          case 3: m.left[g] = -1; break;
          case 4: std::swap(m.left[g], m.left[rnd_in(0, (int)m.left.size() - 1)]); break;
          case 5: m.tree_off[rnd_in(0, (int)m.tree_off.size() - 1)] += rnd_in(-2, 2); break;
        }
        TreeSchedule ms;
        const acrobat_trees mv = m.view();
        // tree_off may now point past the arrays: only call the scheduler when it stays inside them
        bool inside = m.tree_off[0] == 0;
        for (size_t t = 0; t + 1 < m.tree_off.size(); ++t) inside = inside && m.tree_off[t + 1] >= m.tree_off[t];
        inside = inside && m.tree_off.back() <= (int)m.left.size();
        if (!inside && m.tree_off[0] == 0 && m.tree_off.back() > (int)m.left.size()) continue;
        const int rc = schedule_trees(mv, 50, ms, err);
        CHECK(rc == ACROBAT_OK || rc == ACROBAT_EINVAL || rc == ACROBAT_ESTRUCT);
        if (rc == ACROBAT_OK) check_tree_schedule(m, ms);
        const int rc2 = reuse.begin(mv, 50, kept, &toks, err);
        CHECK(rc2 == rc);
        if (rc2 == ACROBAT_OK) reuse.finish(mv, kept);
      }
    }
    // sequences
    std::vector<int32_t> len(rnd_in(0, 40));
    for (auto& x : len) x = rnd_in(0, 25);
    SeqSchedule q;
    CHECK(schedule_seqs((int32_t)len.size(), len.data(), q, err) == ACROBAT_OK);
    int64_t total = 0;
    for (int x : len) total += x;
    CHECK(q.n_rows == total && (q.n_levels == 0 || q.level_off.back() == total));
    BirnnSchedule bs;
    CHECK(schedule_birnn((int32_t)len.size(), len.data(), bs, err) == ACROBAT_OK);
    CHECK(bs.n_rows == total && (total == 0 || (int64_t)bs.level_codes.size() == 3 * total));
    if (!len.empty()) {
      len[0] = -3;
      CHECK(schedule_seqs((int32_t)len.size(), len.data(), q, err) == ACROBAT_EINVAL);
    }
  }
  // the tree-generation program without fibers and without a GPU: the structure only
  for (int round = 0; round < 6; ++round) {
    Dfg graph[kMaxTdcGroups];
    Dfg* graphs[kMaxTdcGroups] = {&graph[0], &graph[1]};
    static float none[1];
    const int n_inst = rnd_in(0, 9), n_labels = rnd_in(1, 7), cap = round == 5 ? 3 : 4000;
    DrnnOps ops{};
    for (Dfg& g : graph) {
      acrobat_op_desc cell{};
      cell.epilogue = ACROBAT_EPI_RNN_STEP; cell.H = 32; cell.nseg = 2; cell.kseg = 32; cell.ld0 = cell.ld1 = 32; cell.ldw = 64;
      cell.src0 = cell.src1 = cell.W = none; cell.h = none;
      cell.src0_rows = cell.out_rows = cap; cell.src1_rows = n_labels;
      int32_t* ids[5] = {&ops.a_root, &ops.a, &ops.f_first, &ops.f, &ops.p};
      for (int i = 0; i < 5; ++i) {
        acrobat_op_desc d = cell;
        if (i == 0) d.src0_rows = n_inst > 0 ? n_inst : 1;
        if (i == 2) d.src0_rows = 1;
        if (i == 4) d.src1_rows = cap;
        CHECK(g.register_op(d, ids[i], err) == ACROBAT_OK);
      }
      acrobat_op_desc o{};
      o.epilogue = ACROBAT_EPI_STORE_Z1; o.H = 32; o.nseg = 1; o.kseg = 32; o.ld0 = 32; o.ldw = 32;
      o.src0 = o.W = none; o.zout = none; o.src0_rows = o.out_rows = cap;
      CHECK(g.register_op(o, &ops.o, err) == ACROBAT_OK);
    }
    acrobat_drnn_decisions dec{};
    dec.seed = 1234 + round; dec.max_depth = 5; dec.max_children = 3; dec.p_child = 0.7f; dec.p_sibling = 0.6f;
    DfgBuckets buckets;
    const DrnnEvaluate evaluate = [&](int32_t group, size_t first, int32_t* n_buckets) {
      graph[group].bucket(buckets, first);
      *n_buckets = (int32_t)buckets.op.size();
      return ACROBAT_OK;
    };
    const DrnnWait wait = [](int32_t) { return ACROBAT_OK; };
    const DrnnScores scores = [](int32_t) { return (const float*)nullptr; };
    DrnnTrees t;
    DrnnStats st;
    const int rc = drnn_generate(graphs, 1, ops, n_inst, n_labels, 32, dec, ACROBAT_TDC_SEQUENTIAL, (round & 1) != 0, cap, evaluate,
                                 wait, scores, t, st, err);
    CHECK(rc == ACROBAT_OK || (rc == ACROBAT_ENOMEM && cap == 3));
    CHECK(t.inst.size() <= (size_t)cap);
    for (size_t i = 0; i < t.inst.size(); ++i) CHECK(t.parent[i] < (int)i && t.label[i] >= 0 && t.label[i] < n_labels);
  }
  std::printf("host code under the sanitizers: ok\n");
  return 0;
}
