// Host level scheduler.
//
// Depth schedule of section 4.1: a node that consumes nothing produced inside the graph
// has depth 0, any other node 1 + the largest depth among its producers; batches run by
// increasing depth and the members of one depth are independent.  One schedule node is a
// whole cell (appendix "Grain Size Coarsening"), every leaf cell only consumes its embedding row so all leaves
// land in depth 0 (the hoisted input transform of appendix "Operator Hoisting"), and sibling subtrees are
// concurrent (section 4.1, "instance parallelism").
//
// The paper computes depths inline while the unbatched program runs, relying on program
// order being a valid dependency order.  Here the structure arrives as index arrays in an
// arbitrary numbering, so depths are propagated upwards from the leaves through parent links
// (one pass, O(N)), which also detects malformed input; a counting sort by depth then
// produces the per-level lists.
#include "scheduler.h"

#include <algorithm>
#include <limits>

namespace acrobat {

namespace {
std::string at_node(const char* what, int32_t tree, int32_t local) {
  return std::string(what) + " (tree " + std::to_string(tree) + ", node " + std::to_string(local) + ")";
}
}  // namespace

// One tree whose numbering is arbitrary: parents are recorded first, then depths are pushed upwards from the
// leaves; a node is final once both children are.  Detects every malformation, cycles included.
int TreeScheduler::general_tree(const acrobat_trees& tr, int32_t t, int32_t vocab, std::string& err) {
  const int32_t base = tr.tree_off[t], n = tr.tree_off[t + 1] - base;
  int32_t* parent = parent_.data();
  int32_t* depth = depth_.data();
  uint8_t* pending = mark_.data();
  for (int32_t j = 0; j < n; ++j) {
    parent[base + j] = -1;
    depth[base + j] = 0;
    pending[base + j] = 0;
  }
  for (int32_t j = 0; j < n; ++j) {
    const int32_t l = tr.left[base + j], r = tr.right[base + j];
    if (l == -1 && r == -1) {
      if (vocab >= 0) {
        const int32_t tok = tr.token[base + j];
        if (tok < 0 || tok >= vocab) { err = at_node("leaf token out of range", t, j); return ACROBAT_ESTRUCT; }
      }
      continue;
    }
    if (l < 0 || r < 0) {
      err = at_node((l < -1 || r < -1) ? "child index out of range" : "node has exactly one child", t, j);
      return ACROBAT_ESTRUCT;
    }
    if (l >= n || r >= n) { err = at_node("child index out of range", t, j); return ACROBAT_ESTRUCT; }
    if (l == j || r == j) { err = at_node("node is its own child", t, j); return ACROBAT_ESTRUCT; }
    if (l == r) { err = at_node("both children are the same node", t, j); return ACROBAT_ESTRUCT; }
    if (parent[base + l] != -1) { err = at_node("node has two parents", t, l); return ACROBAT_ESTRUCT; }
    parent[base + l] = base + j;
    if (parent[base + r] != -1) { err = at_node("node has two parents", t, r); return ACROBAT_ESTRUCT; }
    parent[base + r] = base + j;
    pending[base + j] = 2;
  }
  int32_t roots = 0;
  for (int32_t j = 0; j < n; ++j) roots += parent[base + j] == -1;
  if (roots != 1) {
    err = "tree " + std::to_string(t) + " has " + std::to_string(roots) + " roots (need exactly 1)";
    return ACROBAT_ESTRUCT;
  }
  int32_t done = 0;
  for (int32_t j = 0; j < n; ++j) {
    if (tr.left[base + j] >= 0) continue;
    int32_t g = base + j;  // a leaf: walk up while we complete parents
    ++done;
    while (true) {
      const int32_t p = parent[g];
      if (p < 0) break;
      depth[p] = std::max(depth[p], depth[g] + 1);
      if (--pending[p]) break;
      ++done;
      g = p;
    }
  }
  if (done != n) { err = "tree " + std::to_string(t) + " contains a cycle"; return ACROBAT_ESTRUCT; }
  return ACROBAT_OK;
}

int TreeScheduler::begin(const acrobat_trees& tr, int32_t vocab, TreeSchedule& out, std::vector<int32_t>* leaf_tokens,
                         std::string& err) {
  out.n_nodes = 0;
  out.n_levels = 0;
  out.level_off.assign(1, 0);
  if (tr.n_trees < 0) { err = "n_trees is negative"; return ACROBAT_EINVAL; }
  if (!tr.tree_off) { err = "tree_off is null"; return ACROBAT_EINVAL; }
  if (tr.tree_off[0] != 0) { err = "tree_off[0] must be 0"; return ACROBAT_EINVAL; }
  for (int32_t t = 0; t < tr.n_trees; ++t)
    if (tr.tree_off[t + 1] < tr.tree_off[t]) { err = "tree_off is decreasing"; return ACROBAT_EINVAL; }
  const int32_t N = tr.tree_off[tr.n_trees];
  out.n_nodes = N;
  if (N == 0) {
    out.level_nodes.clear(); out.lrow.clear(); out.rrow.clear();
    if (leaf_tokens) leaf_tokens->clear();
    return ACROBAT_OK;
  }
  if (!tr.left || !tr.right) { err = "left/right is null"; return ACROBAT_EINVAL; }
  if ((vocab >= 0 || leaf_tokens) && !tr.token) { err = "token is null"; return ACROBAT_EINVAL; }

  depth_.resize(N);
  parent_.resize(N);
  mark_.resize(N);
  out.level_nodes.resize(N);
  out.lrow.resize(N);
  out.rrow.resize(N);
  if (leaf_tokens) leaf_tokens->resize(N);
  int32_t* depth = depth_.data();
  uint8_t* claimed = mark_.data();
  int32_t* leaves = out.level_nodes.data();
  int32_t* toks = leaf_tokens ? leaf_tokens->data() : nullptr;
  count_.assign(64, 0);  // nodes per depth, grown on demand
  int32_t n_leaf = 0, max_depth = 0;
  for (int32_t t = 0; t < tr.n_trees; ++t) {
    const int32_t base = tr.tree_off[t], n = tr.tree_off[t + 1] - base;
    if (n == 0) continue;
    // Fast path: a numbering in which every child precedes its parent (what leaves-first / post-order
    // numberings give) cannot hold a cycle, and one ascending pass validates, finds depths and lists leaves.
    // roots = n - 2 * internal nodes once no node has been claimed twice.
    const int32_t* L = tr.left + base;
    const int32_t* R = tr.right + base;
    int32_t* d = depth + base;
    uint8_t* c = claimed + base;
    std::fill(c, c + n, (uint8_t)0);
    const int32_t leaf_mark = n_leaf;
    bool ordered = true;
    int32_t internal = 0;
    for (int32_t j = 0; j < n; ++j) {
      const int32_t l = L[j], r = R[j];
      if ((l & r) == -1) {  // both -1
        if (vocab >= 0) {
          const int32_t tok = tr.token[base + j];
          if (tok < 0 || tok >= vocab) { err = at_node("leaf token out of range", t, j); return ACROBAT_ESTRUCT; }
        }
        d[j] = 0;
        if (toks) toks[n_leaf] = tr.token[base + j];
        leaves[n_leaf++] = base + j;
        continue;
      }
      // unsigned compares: a negative index is "not below j" as well and is sorted out by the general path
      if ((uint32_t)l >= (uint32_t)j || (uint32_t)r >= (uint32_t)j || l == r || (c[l] | c[r])) { ordered = false; break; }
      c[l] = c[r] = 1;
      const int32_t dj = 1 + std::max(d[l], d[r]);
      d[j] = dj;
      max_depth = std::max(max_depth, dj);
      ++internal;
    }
    if (ordered && n - 2 * internal != 1) ordered = false;  // let the general path name the problem
    if (!ordered) {
      n_leaf = leaf_mark;
      const int rc = general_tree(tr, t, vocab, err);
      if (rc != ACROBAT_OK) return rc;
      for (int32_t j = 0; j < n; ++j) {
        if (L[j] < 0) {
          if (toks) toks[n_leaf] = tr.token[base + j];
          leaves[n_leaf++] = base + j;
        }
        max_depth = std::max(max_depth, d[j]);
      }
    }
  }
  // level sizes
  if ((size_t)max_depth + 2 > count_.size()) count_.resize((size_t)max_depth + 2);
  std::fill(count_.begin(), count_.end(), 0);
  for (int32_t g = 0; g < N; ++g) ++count_[depth[g]];
  out.n_levels = max_depth + 1;
  out.level_off.resize((size_t)out.n_levels + 1);
  out.level_off[0] = 0;
  for (int32_t k = 0; k < out.n_levels; ++k) out.level_off[k + 1] = out.level_off[k] + count_[k];
  std::fill(out.lrow.begin(), out.lrow.begin() + n_leaf, -1);
  std::fill(out.rrow.begin(), out.rrow.begin() + n_leaf, -1);
  if (leaf_tokens) leaf_tokens->resize(n_leaf);
  return ACROBAT_OK;
}

void TreeScheduler::finish(const acrobat_trees& tr, TreeSchedule& out) {
  const int32_t N = out.n_nodes;
  if (N == 0 || out.n_levels <= 1) return;
  // counting sort by depth; visiting ids in ascending order keeps each level ascending
  cursor_.assign(out.level_off.begin(), out.level_off.end() - 1);
  const int32_t* depth = depth_.data();
  int32_t* cursor = cursor_.data();
  int32_t* nodes = out.level_nodes.data();
  int32_t* lrow = out.lrow.data();
  int32_t* rrow = out.rrow.data();
  for (int32_t t = 0; t < tr.n_trees; ++t) {
    const int32_t base = tr.tree_off[t];
    for (int32_t g = base; g < tr.tree_off[t + 1]; ++g) {
      const int32_t l = tr.left[g];
      if (l < 0) continue;  // leaves are already listed
      const int32_t pos = cursor[depth[g]]++;
      nodes[pos] = g;
      lrow[pos] = base + l;
      rrow[pos] = base + tr.right[g];
    }
  }
}

int schedule_trees(const acrobat_trees& tr, int32_t vocab, TreeSchedule& out, std::string& err) {
  TreeScheduler s;
  const int rc = s.begin(tr, vocab, out, nullptr, err);
  if (rc != ACROBAT_OK) {
    out = TreeSchedule();
    return rc;
  }
  s.finish(tr, out);
  return ACROBAT_OK;
}

int schedule_seqs(int32_t n_seq, const int32_t* len, SeqSchedule& out, std::string& err) {
  out = SeqSchedule();
  out.level_off.assign(1, 0);
  if (n_seq < 0) { err = "n_seq is negative"; return ACROBAT_EINVAL; }
  if (n_seq == 0) return ACROBAT_OK;
  if (!len) { err = "len is null"; return ACROBAT_EINVAL; }
  int64_t total = 0;
  int32_t tmax = 0;
  for (int32_t s = 0; s < n_seq; ++s) {
    if (len[s] < 0) { err = "negative sequence length at " + std::to_string(s); return ACROBAT_EINVAL; }
    total += len[s];
    tmax = std::max(tmax, len[s]);
  }
  if (total > std::numeric_limits<int32_t>::max()) { err = "more than 2^31-1 rows"; return ACROBAT_EINVAL; }
  out.n_rows = total;
  out.n_levels = tmax;
  out.level_off.assign(tmax + 1, 0);
  out.level_rows.resize(static_cast<size_t>(total));
  // active sequences (ascending s) with their first row; filtered in place as steps run out
  std::vector<int32_t> act_seq, act_row0;
  act_seq.reserve(n_seq);
  act_row0.reserve(n_seq);
  int32_t row0 = 0;
  for (int32_t s = 0; s < n_seq; ++s) {
    if (len[s] > 0) { act_seq.push_back(s); act_row0.push_back(row0); }
    row0 += len[s];
  }
  int32_t pos = 0;
  for (int32_t t = 0; t < tmax; ++t) {
    size_t keep = 0;
    for (size_t a = 0; a < act_seq.size(); ++a) {
      if (len[act_seq[a]] > t) {
        out.level_rows[pos++] = act_row0[a] + t;
        act_seq[keep] = act_seq[a];
        act_row0[keep] = act_row0[a];
        ++keep;
      }
    }
    act_seq.resize(keep);
    act_row0.resize(keep);
    out.level_off[t + 1] = pos;
  }
  return ACROBAT_OK;
}

int schedule_birnn(int32_t n_seq, const int32_t* len, BirnnSchedule& out, std::string& err) {
  out = BirnnSchedule();
  out.level_off.assign(1, 0);
  out.fwd_off.assign(1, 0);
  SeqSchedule f;
  const int rc = schedule_seqs(n_seq, len, f, err);  // forward recurrence: step k = time k
  if (rc != ACROBAT_OK) return rc;
  const int64_t R = f.n_rows;
  if (R == 0) return ACROBAT_OK;
  if (3 * R > std::numeric_limits<int32_t>::max()) { err = "more than (2^31-1)/3 rows"; return ACROBAT_EINVAL; }
  out.n_rows = R;
  out.n_levels = f.n_levels + 1;
  out.level_off.assign(out.n_levels + 1, 0);
  out.fwd_off.assign(f.n_levels + 1, 0);
  out.level_codes.resize(static_cast<size_t>(3 * R));
  // last row of every sequence, by the sequence's first row (for the mirrored backward step)
  std::vector<int32_t> last_of_first(static_cast<size_t>(R), 0);
  {
    int32_t row0 = 0;
    for (int32_t s = 0; s < n_seq; ++s) {
      if (len[s] > 0) last_of_first[row0] = row0 + len[s] - 1;
      row0 += len[s];
    }
  }
  int32_t pos = 0;
  for (int32_t k = 0; k < f.n_levels; ++k) {
    const int32_t b = f.level_off[k], e = f.level_off[k + 1];
    for (int32_t p = b; p < e; ++p) out.level_codes[pos++] = f.level_rows[p];  // forward: row0 + k
    for (int32_t p = b; p < e; ++p) {                                          // backward: last - k
      const int32_t row0 = f.level_rows[p] - k;
      out.level_codes[pos++] = static_cast<int32_t>(R) + last_of_first[row0] - k;
    }
    out.fwd_off[k + 1] = out.fwd_off[k] + (e - b);
    out.level_off[k + 1] = pos;
  }
  for (int32_t r = 0; r < R; ++r) out.level_codes[pos++] = static_cast<int32_t>(2 * R) + r;
  out.level_off[out.n_levels] = pos;
  return ACROBAT_OK;
}

}  // namespace acrobat
