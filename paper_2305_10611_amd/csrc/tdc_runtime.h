// Programs with tensor-dependent control flow on the batched dataflow-graph runtime (section 4.2),
// and the one such program this library ships: top-down tree generation with a doubly recurrent
// network (table 3; evaluated in Evaluation, "Overall Performance" with emulated decisions).
//
// The unbatched program is ordinary recursive code that calls invoke() for every operator, with
// the depth it computes inline, and await() wherever it needs a tensor's value to decide how to
// go on.  Each instance runs on a fiber, and (mode FORK_JOIN) so does every list of children,
// since the subtrees of a node can be generated independently of each other.  When every fiber
// waits, the operators invoked since the last evaluation are executed in batches and the fibers
// go on.  Host code only: the evaluation itself is a callback.
#pragma once
#include <cstdint>
#include <functional>
#include <string>
#include <vector>

#include "acrobat.h"
#include "dfg_runtime.h"

namespace acrobat {

struct DrnnOps {  // ids of the ops registered in the graph
  int32_t a_root, a, f_first, f, p, o;
};

struct DrnnTrees {  // one entry per generated node, in the order of creation
  std::vector<int32_t> inst, parent, prev, sib_index, depth, label, round;
};

struct DrnnStats {
  int32_t n_rounds = 0;    // evaluations (of the group that needed most)
  int32_t n_buckets = 0;   // batches over all evaluations
  int32_t n_fibers = 0;    // fibers started
  int32_t n_ghosts = 0;    // ghost operations invoked
};

// The decisions of one node.  Emulated from its position (the paper's evaluation replaces the
// tensor-dependent decisions by pseudo-random ones since its models are untrained, Evaluation, "Overall Performance") or,
// with dec.from_scores, read off `y`, the node's n_out scores on the host - the value the program
// had to wait for either way.
struct DrnnDecision { bool has_child, has_sibling; int32_t label; };
uint64_t drnn_root_key(uint64_t seed, int32_t inst);
uint64_t drnn_child_key(uint64_t parent_key, int32_t k);
DrnnDecision drnn_decide(const acrobat_drnn_decisions& d, int32_t n_labels, int32_t n_out, uint64_t key, int32_t depth,
                         int32_t k, bool is_root, const float* y);

// The instances are dealt out to n_groups groups (instance s to group s % n_groups), each with a
// graph and a set of fibers of its own.  While one group's operators execute, the host runs the
// program of the other: the two never wait at the same time (with one group the host and the device
// simply alternate).
//   evaluate(group, first_graph_node, &n_buckets)  starts the execution of that group's graph nodes
//     from first_graph_node on and returns without waiting;
//   wait(group)  returns when everything started for the group has finished; the scores of its nodes
//     are then readable through scores(node) (which may return null when nothing is computed at all).
using DrnnEvaluate = std::function<int(int32_t, size_t, int32_t*)>;
using DrnnWait = std::function<int(int32_t)>;
using DrnnScores = std::function<const float*(int32_t)>;

constexpr int32_t kMaxTdcGroups = 2;
// Two groups pay once the host program of an evaluation takes longer than issuing its launches a
// second time (measured: from about 200 instances on, 4 % at 256, 18 % at 1024; below, the host is
// busier with two groups than it was idle with one).
inline int32_t drnn_default_groups(int32_t n_inst, int32_t mode) {
  return mode != ACROBAT_TDC_SEQUENTIAL && n_inst >= 192 ? kMaxTdcGroups : 1;
}

// Runs the generation program for n_inst instances.  graphs[0 .. n_groups): one graph per group, the
// operators registered alike in each.  mode: ACROBAT_TDC_* (without fibers there is one group).
// use_ghosts: align the ancestral cell of a later sibling with its fraternal cell by a ghost
// operation.  Fails with ACROBAT_ENOMEM when more than max_nodes nodes would be generated.
int drnn_generate(Dfg* const* graphs, int32_t n_groups, const DrnnOps& ops, int32_t n_inst, int32_t n_labels, int32_t n_out,
                  const acrobat_drnn_decisions& dec, int32_t mode, bool use_ghosts, int32_t max_nodes,
                  const DrnnEvaluate& evaluate, const DrnnWait& wait, const DrnnScores& scores, DrnnTrees& out,
                  DrnnStats& stats, std::string& err);

}  // namespace acrobat
