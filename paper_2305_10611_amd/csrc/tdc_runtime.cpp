#include "tdc_runtime.h"

#include <algorithm>

#include "fiber.h"

namespace acrobat {

namespace {

// One step of the splitmix64 sequence from state z.
uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

double unit_interval(uint64_t bits) { return (double)(bits >> 11) * (1.0 / 9007199254740992.0); }

// The generation program and the state it shares across its fibers.
struct Generator {
  Dfg& g;
  const DrnnOps& ops;
  const int32_t n_labels, n_out;
  const acrobat_drnn_decisions& dec;
  const bool fork, use_ghosts;
  const int32_t max_nodes;
  const DrnnEvaluate& evaluate;
  const DrnnScores& scores;
  DrnnTrees& out;
  DrnnStats& stats;
  std::string& err;
  FiberScheduler* fibers;  // null: no fibers, every await evaluates at once

  std::vector<int32_t> o_node, o_depth;  // per tree node: graph node and depth of its score operator
  std::vector<int32_t> f_rows;           // per tree node: row holding its fraternal state (0 for first children)
  std::vector<int32_t> deferred;         // first children whose own fraternal row is still to be written
  int32_t first_f_node = -1;             // graph node that computes the shared first-child fraternal state
  size_t executed = 0;                   // graph nodes [0, executed) have been evaluated
  int32_t scored = 0;                    // tree nodes [0, scored) have their scores
  int rc = ACROBAT_OK;

  bool failed() const { return rc != ACROBAT_OK; }
  void fail(int code, const std::string& msg) {
    if (rc == ACROBAT_OK) { rc = code; err = msg; }
  }

  // executes everything invoked since the last evaluation (counts_as_round false: the deferred
  // batch at the end, which no decision waits for)
  void evaluate_pending(bool counts_as_round = true) {
    if (failed() || executed == g.size()) return;
    const int32_t n_new = (int32_t)out.inst.size() - scored;
    int32_t buckets = 0;
    const int e = evaluate(executed, scored, n_new, &buckets);
    if (e != ACROBAT_OK) { fail(e, err.empty() ? "evaluation failed" : err); return; }
    for (int32_t i = scored; i < scored + n_new; ++i) out.round[i] = stats.n_rounds;
    executed = g.size();
    scored += n_new;
    stats.n_buckets += buckets;
    if (counts_as_round) ++stats.n_rounds;
  }

  // returns once the scores of tree node i exist
  void await(int32_t i) {
    if (failed() || (size_t)o_node[i] < executed) return;
    if (fibers && fibers->in_fiber()) fibers->block();  // the scheduler evaluates when nobody can go on
    else evaluate_pending();
  }

  // One node: the three cells and the score layer, each invoked with its depth computed inline.
  // parent / prev: tree nodes or -1.  Returns the tree node, -1 after a failure.
  //
  // The fraternal state of a first child depends on nothing but the parameters (no previous
  // sibling: zero state, label 0): it is the same vector for every first child and for every root.
  // As the paper does for constant tensors (section 7.2), it is computed once - with the roots, in
  // the first evaluation - and reused: consumers of a first child's fraternal state read the row of
  // tree node 0 instead.  The first children's own rows of the output are filled by one batch at the
  // very end (deferred), off the chain of dependent evaluations.
  int32_t node(int32_t inst, int32_t parent, int32_t prev, int32_t k, int32_t depth) {
    if (failed()) return -1;
    const int32_t i = (int32_t)out.inst.size();
    if (i >= max_nodes) { fail(ACROBAT_ENOMEM, "more nodes generated than max_nodes"); return -1; }
    int32_t d_a = parent >= 0 ? o_depth[parent] + 1 : 0;
    int32_t prod_a = parent >= 0 ? o_node[parent] : -1;
    const int32_t d_f = prev >= 0 ? o_depth[prev] + 1 : d_a;  // a first child's fraternal cell waits for nothing
    if (use_ghosts && d_a < d_f) {
      // the parent's scores are older than the previous sibling's: without a ghost the ancestral
      // cells of first, second, third ... children would sit at different depths, one batch each
      if (g.ghost(0, d_f - 1, prod_a, &prod_a, err) != ACROBAT_OK) { fail(ACROBAT_EINVAL, err); return -1; }
      ++stats.n_ghosts;
      d_a = d_f;
    }
    int32_t n_a = -1, n_f = -1, n_p = -1, n_o = -1;
    int32_t f_row = i;  // row of the fraternal arena that holds this node's fraternal state
    int e;
    if (parent >= 0) e = g.invoke(ops.a, 0, d_a, i, parent, out.label[parent], prod_a, -1, &n_a, err);
    else e = g.invoke(ops.a_root, 0, d_a, i, inst, 0, -1, -1, &n_a, err);
    if (e == ACROBAT_OK) {
      if (prev >= 0) {
        e = g.invoke(ops.f, 0, d_f, i, f_rows[prev], out.label[prev], o_node[prev], -1, &n_f, err);
      } else if (parent < 0) {
        e = g.invoke(ops.f_first, 0, d_f, i, 0, 0, -1, -1, &n_f, err);
        if (i == 0) first_f_node = n_f;
      } else {
        f_row = 0;
        n_f = first_f_node;
        deferred.push_back(i);
      }
    }
    const int32_t d_p = std::max(d_a, d_f) + 1;
    if (e == ACROBAT_OK) e = g.invoke(ops.p, 0, d_p, i, i, f_row, n_a, n_f, &n_p, err);
    if (e == ACROBAT_OK) e = g.invoke(ops.o, 0, d_p + 1, i, i, 0, n_p, -1, &n_o, err);
    if (e != ACROBAT_OK) { fail(e, err); return -1; }
    out.inst.push_back(inst);
    out.parent.push_back(parent);
    out.prev.push_back(prev);
    out.sib_index.push_back(k);
    out.depth.push_back(depth);
    out.label.push_back(-1);
    out.round.push_back(-1);
    o_node.push_back(n_o);
    o_depth.push_back(d_p + 1);
    f_rows.push_back(f_row);
    return i;
  }

  // the deferred batch: the first children's own fraternal rows
  void finish() {
    if (failed() || deferred.empty()) return;
    for (int32_t i : deferred)
      if (g.invoke(ops.f_first, 0, 0, i, 0, 0, -1, -1, nullptr, err) != ACROBAT_OK) { fail(ACROBAT_EINVAL, err); return; }
    evaluate_pending(false);
  }

  // the children of `parent`, left to right.  The subtree under a child that has a next sibling is
  // generated by a fiber of its own (fork) while this one goes on with the siblings; under the last
  // child this fiber simply descends - nothing is left for it to do at this level.
  void children(int32_t inst, int32_t parent, uint64_t pkey, int32_t pdepth) {
    for (;;) {  // one level per turn
      int32_t prev = -1, last = -1;
      uint64_t last_key = 0;
      for (int32_t k = 0;; ++k) {
        const uint64_t key = drnn_child_key(pkey, k);
        const int32_t i = node(inst, parent, prev, k, pdepth + 1);
        if (i < 0) return;
        await(i);
        if (failed()) return;
        const DrnnDecision d = drnn_decide(dec, n_labels, n_out, key, pdepth + 1, k, false, scores(i));
        out.label[i] = d.label;
        if (d.has_child) {
          if (d.has_sibling && fork && fibers) {
            spawn_children(inst, i, key, pdepth + 1);
          } else if (d.has_sibling) {
            children(inst, i, key, pdepth + 1);  // no fibers for subtrees: depth first
          } else {
            last = i;
            last_key = key;
          }
        }
        if (failed() || !d.has_sibling) break;
        prev = i;
      }
      if (failed() || last < 0) return;
      parent = last;
      pkey = last_key;
      ++pdepth;
    }
  }

  struct ForkArgs { Generator* gen; int32_t inst, parent, pdepth; uint64_t pkey; };
  static void fork_entry(void* p) {
    const ForkArgs a = *static_cast<const ForkArgs*>(p);
    a.gen->children(a.inst, a.parent, a.pkey, a.pdepth);
  }
  void spawn_children(int32_t inst, int32_t parent, uint64_t pkey, int32_t pdepth) {
    ++stats.n_fibers;
    const ForkArgs a{this, inst, parent, pdepth, pkey};
    if (!fibers->spawn(&fork_entry, &a, sizeof(a))) fail(ACROBAT_ENOMEM, "no memory for a fiber stack");
  }

  void instance(int32_t inst) {
    const uint64_t key = drnn_root_key(dec.seed, inst);
    const int32_t i = node(inst, -1, -1, 0, 0);
    if (i < 0) return;
    await(i);
    if (failed()) return;
    const DrnnDecision d = drnn_decide(dec, n_labels, n_out, key, 0, 0, true, scores(i));
    out.label[i] = d.label;
    if (d.has_child) children(inst, i, key, 0);  // a root has no siblings: its fiber descends itself
  }
};

}  // namespace

uint64_t drnn_root_key(uint64_t seed, int32_t inst) { return mix64(seed ^ mix64((uint64_t)inst)); }
uint64_t drnn_child_key(uint64_t parent_key, int32_t k) { return mix64(parent_key + (uint64_t)k + 1u); }

DrnnDecision drnn_decide(const acrobat_drnn_decisions& d, int32_t n_labels, int32_t n_out, uint64_t key, int32_t depth,
                         int32_t k, bool is_root, const float* y) {
  DrnnDecision r;
  if (d.from_scores) {
    r.has_child = depth + 1 < d.max_depth && y[0] > 0.0f;
    r.has_sibling = !is_root && k + 1 < d.max_children && y[1] > 0.0f;
    const int32_t n = n_labels < n_out - 2 ? n_labels : n_out - 2;
    r.label = 0;
    for (int32_t l = 1; l < n; ++l)
      if (y[2 + l] > y[2 + r.label]) r.label = l;
    return r;
  }
  // the emulation does not look at the scores it waited for
  r.has_child = depth + 1 < d.max_depth && unit_interval(mix64(key ^ 1u)) < (double)d.p_child;
  r.has_sibling = !is_root && k + 1 < d.max_children && unit_interval(mix64(key ^ 2u)) < (double)d.p_sibling;
  r.label = (int32_t)(mix64(key ^ 3u) % (uint64_t)n_labels);
  return r;
}

int drnn_generate(Dfg& g, const DrnnOps& ops, int32_t n_inst, int32_t n_labels, int32_t n_out, const acrobat_drnn_decisions& dec,
                  int32_t mode, bool use_ghosts, int32_t max_nodes, const DrnnEvaluate& evaluate,
                  const DrnnScores& scores, DrnnTrees& out, DrnnStats& stats, std::string& err) {
  out = DrnnTrees();
  stats = DrnnStats();
  if (n_inst < 0 || n_labels < 1 || max_nodes < 0 || dec.max_depth < 1 || dec.max_children < 1 ||
      (!dec.from_scores && (!(dec.p_child >= 0.0f && dec.p_child <= 1.0f) || !(dec.p_sibling >= 0.0f && dec.p_sibling <= 1.0f))) ||
      (dec.from_scores && n_out < 3)) {
    err = "bad generation parameters";
    return ACROBAT_EINVAL;
  }
  if (mode != ACROBAT_TDC_SEQUENTIAL && mode != ACROBAT_TDC_INSTANCE_FIBERS && mode != ACROBAT_TDC_FORK_JOIN) {
    err = "unknown mode";
    return ACROBAT_EINVAL;
  }
  // the recursion over a tree's levels runs on a fiber's stack (or, without fibers, on the caller's)
  if (dec.max_depth > 4096) {
    err = "max_depth above 4096";
    return ACROBAT_EINVAL;
  }
  FiberScheduler fibers(((size_t)64 << 10) + ((size_t)1 << 10) * (size_t)dec.max_depth);
  Generator gen{g, ops, n_labels, n_out, dec, mode == ACROBAT_TDC_FORK_JOIN, use_ghosts, max_nodes, evaluate, scores, out, stats, err,
                mode == ACROBAT_TDC_SEQUENTIAL ? nullptr : &fibers};
  if (mode == ACROBAT_TDC_SEQUENTIAL) {
    for (int32_t s = 0; s < n_inst && !gen.failed(); ++s) gen.instance(s);
    gen.finish();
    return gen.rc;
  }
  for (int32_t s = 0; s < n_inst; ++s) {
    ++stats.n_fibers;
    struct Args { Generator* gen; int32_t inst; } a{&gen, s};
    if (!fibers.spawn([](void* p) { const Args x = *static_cast<const Args*>(p); x.gen->instance(x.inst); }, &a, sizeof(a))) {
      err = "no memory for a fiber stack";
      return ACROBAT_ENOMEM;
    }
  }
  // all fibers advance until each has finished or waits for scores; then one evaluation for all
  for (;;) {
    fibers.run();
    if (fibers.blocked() == 0) break;
    gen.evaluate_pending();  // (after a failure: nothing; the released fibers see it and return)
    fibers.release();
  }
  if (!gen.failed() && !fibers.error().empty()) gen.fail(ACROBAT_EINVAL, "exception in a fiber: " + fibers.error());
  gen.finish();
  return gen.rc;
}

}  // namespace acrobat
