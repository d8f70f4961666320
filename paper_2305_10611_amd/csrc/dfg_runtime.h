// Generic batched-dataflow-graph runtime (host side): the unbatched program of one mini-batch
// calls invoke(op, phase, depth, ...) once per operator instance, with the depth it computed
// inline (section 4.1, listing 2); run() executes the graph bucket by bucket, a bucket being all
// nodes of one (phase, depth, op).  New cells need an op description, not a scheduler.
#pragma once
#include <cstdint>
#include <initializer_list>
#include <string>
#include <vector>

#include "acrobat.h"

namespace acrobat {

struct DfgNode {
  int32_t op, phase, depth;  // op < 0: a ghost operation (holds a depth, launches nothing)
  int32_t out_row, arg0, arg1;
};

struct DfgBuckets {
  std::vector<int32_t> off;    // [n_buckets + 1] into order
  std::vector<int32_t> order;  // node ids: (phase, depth, op) ascending, node id ascending inside
  std::vector<int32_t> op;     // [n_buckets] op of each bucket
};

class Dfg {
 public:
  int register_op(const acrobat_op_desc& d, int32_t* id, std::string& err);
  void clear() { nodes_.clear(); }
  size_t size() const { return nodes_.size(); }
  // prod0 / prod1: node ids of the producers of the operands (-1: an input of the graph).  The
  // inline depth is checked against them: a node must be deeper than every producer of its own phase
  // and must not be in an earlier phase than a producer.
  int invoke(int32_t op, int32_t phase, int32_t depth, int32_t out_row, int32_t arg0, int32_t arg1, int32_t prod0,
             int32_t prod1, int32_t* node, std::string& err);
  // A ghost operation (section 4.1, appendix "Combating Eagerness of Depth Scheduling"): a node that only occupies a depth.  A program
  // whose branches reach the same operator after different numbers of steps invokes ghosts on the
  // shorter branch, so that the operator lands at one depth - one batch - for every instance.  It is
  // checked against its producer like any node and can be named as a producer; it is never executed.
  int ghost(int32_t phase, int32_t depth, int32_t prod, int32_t* node, std::string& err);
  // Counting sort of the nodes `first`, `first + 1`, ... into buckets (ghosts left out),
  // O(nodes + phases * depths * ops).  A program with tensor-dependent control flow grows the graph
  // between evaluations; each evaluation buckets the nodes added since the previous one.
  void bucket(DfgBuckets& out, size_t first = 0) const;
  const std::vector<DfgNode>& nodes() const { return nodes_; }
  const std::vector<acrobat_op_desc>& ops() const { return ops_; }

 private:
  int check_depth(int32_t phase, int32_t depth, std::initializer_list<int32_t> producers, std::string& err) const;
  void push(const DfgNode& n, int32_t* node);
  std::vector<acrobat_op_desc> ops_;
  std::vector<DfgNode> nodes_;
  int32_t max_phase_ = 0, max_depth_ = 0;
};

// The unbatched TreeLSTM program written against invoke(): one recursive evaluation per tree
// (explicit stack), a leaf is op_leaf(token) at depth 0 (hoisted), an internal node
// op_internal(left, right) at depth 1 + max(child depths), each node's state goes to arena row
// = its global node id.  Validates the structure as schedule_trees does.
int dfg_build_treelstm(Dfg& g, const acrobat_trees& trees, int32_t vocab, int32_t op_leaf, int32_t op_internal,
                       std::string& err);

}  // namespace acrobat
