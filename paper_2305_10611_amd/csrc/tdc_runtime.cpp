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

// What the groups share: parameters, the forest under construction, the failure state.
struct Shared {
  const DrnnOps& ops;
  const int32_t n_labels, n_out;
  const acrobat_drnn_decisions& dec;
  const bool fork, use_ghosts;
  const int32_t max_nodes;
  const DrnnEvaluate& evaluate;
  const DrnnWait& wait;
  const DrnnScores& scores;
  DrnnTrees& out;
  DrnnStats& stats;
  std::string& err;
  std::vector<int32_t> o_node, o_depth;  // per tree node: graph node (in its group's graph) and depth of its score operator
  std::vector<int32_t> f_rows;           // per tree node: row holding its fraternal state (a shared row for first children)
  std::vector<int32_t> deferred;         // first children whose own fraternal row is still to be written
  int rc = ACROBAT_OK;

  bool failed() const { return rc != ACROBAT_OK; }
  void fail(int code, const std::string& msg) {
    if (rc == ACROBAT_OK) { rc = code; err = msg; }
  }
};

// The generation program of one group of instances and the state its fibers share.
struct Generator {
  Shared& sh;
  Dfg& g;
  const int32_t group;
  FiberScheduler* fibers;  // null: no fibers, every await evaluates at once

  size_t executed = 0;            // graph nodes [0, executed) have been evaluated
  size_t started = 0;             // graph nodes [0, started) have been handed to evaluate()
  std::vector<int32_t> fresh;     // tree nodes created since the last evaluation was started
  std::vector<int32_t> in_flight; // tree nodes of the evaluation that is running
  bool running = false;           // an evaluation has been started and not yet waited for
  int32_t n_evaluations = 0;
  int32_t const_f_row = -1;       // tree node whose fraternal row is the constant first-child state
  int32_t const_f_node = -1;      // graph node that computes it

  bool failed() const { return sh.failed(); }

  // starts the execution of everything invoked since the last evaluation; false: nothing to do
  bool start_evaluation() {
    if (failed() || started == g.size()) return false;
    int32_t buckets = 0;
    const int e = sh.evaluate(group, started, &buckets);
    if (e != ACROBAT_OK) { sh.fail(e, sh.err.empty() ? "evaluation failed" : sh.err); return false; }
    started = g.size();
    in_flight.swap(fresh);
    fresh.clear();
    sh.stats.n_buckets += buckets;
    running = true;
    return true;
  }

  // waits for the running evaluation (counts_as_round false: the deferred batch at the end, which no
  // decision waits for)
  void finish_evaluation(bool counts_as_round = true) {
    if (!running) return;
    running = false;
    const int e = sh.wait(group);
    if (e != ACROBAT_OK) { sh.fail(e, sh.err.empty() ? "evaluation failed" : sh.err); return; }
    for (int32_t i : in_flight) sh.out.round[i] = n_evaluations;
    in_flight.clear();
    executed = started;
    if (counts_as_round) ++n_evaluations;
  }

  // returns once the scores of tree node i exist
  void await(int32_t i) {
    if (failed() || (size_t)sh.o_node[i] < executed) return;
    if (fibers && fibers->in_fiber()) {
      fibers->block();  // the scheduler evaluates when no fiber of the group can go on
    } else if (start_evaluation()) {
      finish_evaluation();
    }
  }

  // One node: the three cells and the score layer, each invoked with its depth computed inline.
  // parent / prev: tree nodes or -1.  Returns the tree node, -1 after a failure.
  //
  // The fraternal state of a first child depends on nothing but the parameters (no previous
  // sibling: zero state, label 0): it is the same vector for every first child and for every root.
  // As the paper does for constant tensors (Evaluation, "Overall Performance"), it is computed once per group - with the
  // roots, in the first evaluation - and reused: consumers of a first child's fraternal state read
  // the row of the group's first root instead.  The first children's own rows of the output are
  // filled by one batch at the very end (deferred), off the chain of dependent evaluations.
  int32_t node(int32_t inst, int32_t parent, int32_t prev, int32_t k, int32_t depth) {
    if (failed()) return -1;
    DrnnTrees& out = sh.out;
    const DrnnOps& ops = sh.ops;
    const int32_t i = (int32_t)out.inst.size();
    if (i >= sh.max_nodes) { sh.fail(ACROBAT_ENOMEM, "more nodes generated than max_nodes"); return -1; }
    int32_t d_a = parent >= 0 ? sh.o_depth[parent] + 1 : 0;
    int32_t prod_a = parent >= 0 ? sh.o_node[parent] : -1;
    const int32_t d_f = prev >= 0 ? sh.o_depth[prev] + 1 : d_a;  // a first child's fraternal cell waits for nothing
    if (sh.use_ghosts && d_a < d_f) {
      // the parent's scores are older than the previous sibling's: without a ghost the ancestral
      // cells of first, second, third ... children would sit at different depths, one batch each
      if (g.ghost(0, d_f - 1, prod_a, &prod_a, sh.err) != ACROBAT_OK) { sh.fail(ACROBAT_EINVAL, sh.err); return -1; }
      ++sh.stats.n_ghosts;
      d_a = d_f;
    }
    int32_t n_a = -1, n_f = -1, n_p = -1, n_o = -1;
    int32_t f_row = i;  // row of the fraternal arena that holds this node's fraternal state
    int e;
    if (parent >= 0) e = g.invoke(ops.a, 0, d_a, i, parent, out.label[parent], prod_a, -1, &n_a, sh.err);
    else e = g.invoke(ops.a_root, 0, d_a, i, inst, 0, -1, -1, &n_a, sh.err);
    if (e == ACROBAT_OK) {
      if (prev >= 0) {
        e = g.invoke(ops.f, 0, d_f, i, sh.f_rows[prev], out.label[prev], sh.o_node[prev], -1, &n_f, sh.err);
      } else if (parent < 0) {
        e = g.invoke(ops.f_first, 0, d_f, i, 0, 0, -1, -1, &n_f, sh.err);
        if (const_f_row < 0) {
          const_f_row = i;
          const_f_node = n_f;
        }
      } else {
        f_row = const_f_row;
        n_f = const_f_node;
        sh.deferred.push_back(i);
      }
    }
    const int32_t d_p = std::max(d_a, d_f) + 1;
    if (e == ACROBAT_OK) e = g.invoke(ops.p, 0, d_p, i, i, f_row, n_a, n_f, &n_p, sh.err);
    if (e == ACROBAT_OK) e = g.invoke(ops.o, 0, d_p + 1, i, i, 0, n_p, -1, &n_o, sh.err);
    if (e != ACROBAT_OK) { sh.fail(e, sh.err); return -1; }
    out.inst.push_back(inst);
    out.parent.push_back(parent);
    out.prev.push_back(prev);
    out.sib_index.push_back(k);
    out.depth.push_back(depth);
    out.label.push_back(-1);
    out.round.push_back(-1);
    sh.o_node.push_back(n_o);
    sh.o_depth.push_back(d_p + 1);
    sh.f_rows.push_back(f_row);
    fresh.push_back(i);
    return i;
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
        const DrnnDecision d = drnn_decide(sh.dec, sh.n_labels, sh.n_out, key, pdepth + 1, k, false, sh.scores(i));
        sh.out.label[i] = d.label;
        if (d.has_child) {
          if (d.has_sibling && sh.fork && fibers) {
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
    ++sh.stats.n_fibers;
    const ForkArgs a{this, inst, parent, pdepth, pkey};
    if (!fibers->spawn(&fork_entry, &a, sizeof(a))) sh.fail(ACROBAT_ENOMEM, "no memory for a fiber stack");
  }

  void instance(int32_t inst) {
    const uint64_t key = drnn_root_key(sh.dec.seed, inst);
    const int32_t i = node(inst, -1, -1, 0, 0);
    if (i < 0) return;
    await(i);
    if (failed()) return;
    const DrnnDecision d = drnn_decide(sh.dec, sh.n_labels, sh.n_out, key, 0, 0, true, sh.scores(i));
    sh.out.label[i] = d.label;
    if (d.has_child) children(inst, i, key, 0);  // a root has no siblings: its fiber descends itself
  }

  struct InstanceArgs { Generator* gen; int32_t inst; };
  static void instance_entry(void* p) {
    const InstanceArgs a = *static_cast<const InstanceArgs*>(p);
    a.gen->instance(a.inst);
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

int drnn_generate(Dfg* const* graphs, int32_t n_groups, const DrnnOps& ops, int32_t n_inst, int32_t n_labels, int32_t n_out,
                  const acrobat_drnn_decisions& dec, int32_t mode, bool use_ghosts, int32_t max_nodes,
                  const DrnnEvaluate& evaluate, const DrnnWait& wait, const DrnnScores& scores, DrnnTrees& out,
                  DrnnStats& stats, std::string& err) {
  out = DrnnTrees();
  stats = DrnnStats();
  if (n_inst < 0 || n_labels < 1 || max_nodes < 0 || dec.max_depth < 1 || dec.max_children < 1 ||
      (!dec.from_scores && (!(dec.p_child >= 0.0f && dec.p_child <= 1.0f) || !(dec.p_sibling >= 0.0f && dec.p_sibling <= 1.0f))) ||
      (dec.from_scores && n_out < 3) || !graphs || n_groups < 1 || n_groups > kMaxTdcGroups) {
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
  Shared sh{ops, n_labels, n_out, dec, mode == ACROBAT_TDC_FORK_JOIN, use_ghosts, max_nodes, evaluate, wait, scores, out, stats, err};
  if (mode == ACROBAT_TDC_SEQUENTIAL) n_groups = 1;
  const size_t stack_bytes = ((size_t)64 << 10) + ((size_t)1 << 10) * (size_t)dec.max_depth;
  FiberScheduler schedulers[kMaxTdcGroups] = {FiberScheduler(stack_bytes), FiberScheduler(stack_bytes)};
  Generator gens[kMaxTdcGroups] = {
      Generator{sh, *graphs[0], 0, mode == ACROBAT_TDC_SEQUENTIAL ? nullptr : &schedulers[0]},
      Generator{sh, *graphs[n_groups > 1 ? 1 : 0], 1, &schedulers[1]}};
  auto finish = [&] {
    // the deferred batch: the first children's own fraternal rows, through the first group's graph
    if (sh.failed() || sh.deferred.empty()) return;
    for (int32_t i : sh.deferred)
      if (gens[0].g.invoke(ops.f_first, 0, 0, i, 0, 0, -1, -1, nullptr, err) != ACROBAT_OK) { sh.fail(ACROBAT_EINVAL, err); return; }
    if (gens[0].start_evaluation()) gens[0].finish_evaluation(false);
  };
  if (mode == ACROBAT_TDC_SEQUENTIAL) {
    for (int32_t s = 0; s < n_inst && !sh.failed(); ++s) gens[0].instance(s);
    finish();
    stats.n_rounds = gens[0].n_evaluations;
    return sh.rc;
  }
  for (int32_t s = 0; s < n_inst; ++s) {
    ++stats.n_fibers;
    Generator& gen = gens[s % n_groups];
    const Generator::InstanceArgs a{&gen, s};
    if (!gen.fibers->spawn(&Generator::instance_entry, &a, sizeof(a))) {
      err = "no memory for a fiber stack";
      return ACROBAT_ENOMEM;
    }
  }
  // Every group: all fibers advance until each has finished or waits for scores, then one evaluation
  // for the group is started.  The host turns to the next group while it runs.
  for (int32_t k = 0; k < n_groups; ++k) {
    gens[k].fibers->run();
    if (gens[k].fibers->blocked() > 0) gens[k].start_evaluation();
  }
  for (bool any = true; any;) {
    any = false;
    for (int32_t k = 0; k < n_groups; ++k) {
      Generator& gen = gens[k];
      if (gen.fibers->blocked() == 0) continue;
      any = true;
      gen.finish_evaluation();  // (after a failure: nothing; the released fibers see it and return)
      gen.fibers->release();
      gen.fibers->run();
      if (gen.fibers->blocked() > 0 && !gen.start_evaluation() && !sh.failed())
        sh.fail(ACROBAT_EINVAL, "fibers wait although nothing is left to evaluate");
    }
  }
  for (int32_t k = 0; k < n_groups; ++k) {
    gens[k].finish_evaluation();
    if (!sh.failed() && !schedulers[k].error().empty()) sh.fail(ACROBAT_EINVAL, "exception in a fiber: " + schedulers[k].error());
    stats.n_rounds = std::max(stats.n_rounds, gens[k].n_evaluations);
  }
  finish();
  return sh.rc;
}

}  // namespace acrobat
