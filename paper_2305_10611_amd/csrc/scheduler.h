// Host level scheduler: structures -> per-depth node lists (no GPU code here).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "acrobat.h"

namespace acrobat {

struct TreeSchedule {
  int32_t n_nodes = 0;
  int32_t n_levels = 0;
  std::vector<int32_t> level_off;    // [n_levels + 1]
  std::vector<int32_t> level_nodes;  // [N] global ids, ascending inside a level
  std::vector<int32_t> lrow, rrow;   // [N] global child ids by list position, -1 at leaves
};

// Returns ACROBAT_OK / EINVAL / ESTRUCT; `err` explains a failure.
int schedule_trees(const acrobat_trees& trees, int32_t vocab, TreeSchedule& out, std::string& err);

// The same schedule in two phases with buffers that live across calls (a context owns one of these), so that
// a forward call can launch level 0 while the host is still sorting the internal levels:
//  begin()  validates the whole structure (nothing may be launched for malformed input), computes every
//           node's depth, level_off, and the level-0 list: out.level_nodes[0 .. n_leaf) = the leaves by
//           ascending id, their tokens in leaf_tokens (if not null; needs trees.token);
//  finish() fills level_nodes / lrow / rrow of the internal levels.
// `out` is resized, never shrunk to fit: its vectors keep their capacity from call to call.
class TreeScheduler {
 public:
  int begin(const acrobat_trees& trees, int32_t vocab, TreeSchedule& out, std::vector<int32_t>* leaf_tokens, std::string& err);
  void finish(const acrobat_trees& trees, TreeSchedule& out);

 private:
  int general_tree(const acrobat_trees& tr, int32_t t, int32_t vocab, std::string& err);
  std::vector<int32_t> depth_, parent_, cursor_, count_;
  std::vector<uint8_t> mark_;  // fast path: "has a parent"; general path: children still to come
};

struct SeqSchedule {
  int64_t n_rows = 0;
  int32_t n_levels = 0;
  std::vector<int32_t> level_off;   // [n_levels + 1]
  std::vector<int32_t> level_rows;  // [sum len]
};

int schedule_seqs(int32_t n_seq, const int32_t* len, SeqSchedule& out, std::string& err);

// Bidirectional RNN with an output phase: levels 0 .. max len - 1 hold step k of both directions
// (codes: forward row, then R + backward row), the last level holds every output operator (2R + row).
struct BirnnSchedule {
  int64_t n_rows = 0;
  int32_t n_levels = 0;              // max len + 1, or 0
  std::vector<int32_t> level_off;    // [n_levels + 1] into level_codes
  std::vector<int32_t> level_codes;  // [3 R]
  std::vector<int32_t> fwd_off;      // [max len + 1]: forward entries of level k are
                                     // level_codes[level_off[k] .. level_off[k] + fwd_off[k+1] - fwd_off[k])
};

int schedule_birnn(int32_t n_seq, const int32_t* len, BirnnSchedule& out, std::string& err);

}  // namespace acrobat
