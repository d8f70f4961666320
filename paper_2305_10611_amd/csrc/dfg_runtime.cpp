#include "dfg_runtime.h"

#include <algorithm>
#include <initializer_list>
#include <limits>

namespace acrobat {

int Dfg::register_op(const acrobat_op_desc& d, int32_t* id, std::string& err) {
  if (d.epilogue < ACROBAT_EPI_TREE_LEAF || d.epilogue > ACROBAT_EPI_MVRNN) { err = "unknown epilogue kind"; return ACROBAT_EINVAL; }
  if (d.epilogue == ACROBAT_EPI_MVRNN) {
    if (d.H != 64 && d.H != 128) { err = "matrix-vector cell: d must be 64 or 128"; return ACROBAT_EINVAL; }
    if (d.nseg != 0) { err = "matrix-vector cell: nseg must be 0"; return ACROBAT_EINVAL; }
    if (!d.src0 || !d.src1 || !d.W || !d.W2 || !d.h || !d.c) { err = "matrix-vector cell: a table, weight or arena pointer is null"; return ACROBAT_EINVAL; }
    if (d.src0_rows <= 0 || d.out_rows <= 0) { err = "row counts must be positive"; return ACROBAT_EINVAL; }
    ops_.push_back(d);
    *id = (int32_t)ops_.size() - 1;
    return ACROBAT_OK;
  }
  if (d.H <= 0 || d.H % 32) { err = "H must be a positive multiple of 32"; return ACROBAT_EINVAL; }
  if (d.nseg < 0 || d.nseg > 2 || (d.nseg > 0 && (d.kseg <= 0 || d.kseg % 32))) { err = "nseg in 0..2, kseg a positive multiple of 32"; return ACROBAT_EINVAL; }
  if (d.nseg > 0 && (!d.src0 || !d.W)) { err = "operand or weight pointer is null"; return ACROBAT_EINVAL; }
  if (d.nseg > 1 && !d.src1) { err = "second operand pointer is null"; return ACROBAT_EINVAL; }
  if (d.epilogue == ACROBAT_EPI_RELU_OUT && (d.n_cols < 1 || d.n_cols > d.H || !d.y)) { err = "output layer: 1 <= n_cols <= H, y not null"; return ACROBAT_EINVAL; }
  const int e = d.epilogue;
  if (d.out_rows <= 0 || (d.nseg > 0 && d.src0_rows <= 0) || (d.nseg > 1 && d.src1_rows <= 0)) { err = "row counts must be positive"; return ACROBAT_EINVAL; }
  if ((e == ACROBAT_EPI_TREE_LEAF || e == ACROBAT_EPI_TREE_INTERNAL || e == ACROBAT_EPI_LSTM_STEP) && (!d.h || !d.c)) { err = "h or c arena is null"; return ACROBAT_EINVAL; }
  if (e == ACROBAT_EPI_TREE_INTERNAL && (!d.cprev_src || d.nseg != 2)) { err = "internal tree cell: two segments and cprev_src"; return ACROBAT_EINVAL; }
  if (e == ACROBAT_EPI_LSTM_STEP && (!d.zadd || (d.cprev_src && d.src0_rows <= 0))) { err = "LSTM step: zadd is null"; return ACROBAT_EINVAL; }
  if (e == ACROBAT_EPI_RNN_STEP && !d.h) { err = "RNN step: h is null"; return ACROBAT_EINVAL; }
  if ((e == ACROBAT_EPI_STORE_Z || e == ACROBAT_EPI_STORE_Z1) && !d.zout) { err = "zout is null"; return ACROBAT_EINVAL; }
  const int gates = d.epilogue == ACROBAT_EPI_TREE_LEAF || d.epilogue == ACROBAT_EPI_TREE_INTERNAL ? 5
                    : d.epilogue == ACROBAT_EPI_LSTM_STEP || d.epilogue == ACROBAT_EPI_STORE_Z ? 4 : 1;
  if ((double)gates * d.H * (double)d.ldw >= 2147483648.0) { err = "weight matrix has 2^31 or more elements"; return ACROBAT_EINVAL; }
  ops_.push_back(d);
  *id = (int32_t)ops_.size() - 1;
  return ACROBAT_OK;
}

int Dfg::check_depth(int32_t phase, int32_t depth, std::initializer_list<int32_t> producers, std::string& err) const {
  if (phase < 0 || depth < 0 || phase > 4096 || depth > (1 << 24)) { err = "phase or depth out of range"; return ACROBAT_EINVAL; }
  if (nodes_.size() >= (size_t)std::numeric_limits<int32_t>::max()) { err = "too many nodes"; return ACROBAT_EINVAL; }
  for (int32_t p : producers) {
    if (p < 0) continue;
    if (p >= (int32_t)nodes_.size()) { err = "producer is not an earlier node"; return ACROBAT_ESTRUCT; }
    const DfgNode& q = nodes_[p];
    if (q.phase > phase || (q.phase == phase && q.depth >= depth)) {
      err = "depth " + std::to_string(depth) + " (phase " + std::to_string(phase) + ") does not come after producer node " +
            std::to_string(p);
      return ACROBAT_ESTRUCT;
    }
  }
  return ACROBAT_OK;
}

void Dfg::push(const DfgNode& n, int32_t* node) {
  if (nodes_.empty()) max_phase_ = max_depth_ = 0;
  max_phase_ = std::max(max_phase_, n.phase);
  max_depth_ = std::max(max_depth_, n.depth);
  nodes_.push_back(n);
  if (node) *node = (int32_t)nodes_.size() - 1;
}

int Dfg::invoke(int32_t op, int32_t phase, int32_t depth, int32_t out_row, int32_t arg0, int32_t arg1, int32_t prod0,
                int32_t prod1, int32_t* node, std::string& err) {
  if (op < 0 || op >= (int32_t)ops_.size()) { err = "unknown op id"; return ACROBAT_EINVAL; }
  if (ops_[op].epilogue == ACROBAT_EPI_MVRNN) {
    const acrobat_op_desc& d = ops_[op];  // children: arena rows, or -(table row + 1)
    if (out_row < 0 || out_row >= d.out_rows || arg0 < -d.src0_rows || arg0 >= d.out_rows || arg1 < -d.src0_rows || arg1 >= d.out_rows) {
      err = "row out of range";
      return ACROBAT_EINVAL;
    }
  } else if (out_row < 0 || arg0 < 0 || arg1 < 0) {
    err = "negative row";
    return ACROBAT_EINVAL;
  } else {
    const acrobat_op_desc& d = ops_[op];
    const bool uses0 = d.nseg > 0 || d.cprev_src, uses1 = d.nseg > 1;
    if (out_row >= d.out_rows || (uses0 && arg0 >= d.src0_rows) || (uses1 && arg1 >= d.src1_rows)) { err = "row out of range"; return ACROBAT_EINVAL; }
  }
  const int rc = check_depth(phase, depth, {prod0, prod1}, err);
  if (rc != ACROBAT_OK) return rc;
  push({op, phase, depth, out_row, arg0, arg1}, node);
  return ACROBAT_OK;
}

int Dfg::ghost(int32_t phase, int32_t depth, int32_t prod, int32_t* node, std::string& err) {
  const int rc = check_depth(phase, depth, {prod}, err);
  if (rc != ACROBAT_OK) return rc;
  push({-1, phase, depth, 0, 0, 0}, node);
  return ACROBAT_OK;
}

void Dfg::bucket(DfgBuckets& out, size_t first) const {
  out.off.assign(1, 0);
  out.order.clear();
  out.op.clear();
  std::vector<int32_t> a, b;
  for (size_t i = first; i < nodes_.size(); ++i)
    if (nodes_[i].op >= 0) a.push_back((int32_t)i);
  const size_t n = a.size();
  if (n == 0) return;
  b.resize(n);
  // three stable counting passes, least significant key first: op, depth, phase
  auto pass = [&](int32_t n_keys, auto key) {
    std::vector<int32_t> cnt((size_t)n_keys + 1, 0);
    for (size_t i = 0; i < n; ++i) ++cnt[(size_t)key(nodes_[a[i]]) + 1];
    for (int32_t k = 0; k < n_keys; ++k) cnt[(size_t)k + 1] += cnt[k];
    for (size_t i = 0; i < n; ++i) b[(size_t)cnt[key(nodes_[a[i]])]++] = a[i];
    a.swap(b);
  };
  // (depths are counted from the smallest one present: late evaluations of a growing graph hold few, deep nodes)
  int32_t dmin = max_depth_;
  for (size_t i = 0; i < n; ++i) dmin = std::min(dmin, nodes_[a[i]].depth);
  pass((int32_t)ops_.size(), [](const DfgNode& x) { return x.op; });
  pass(max_depth_ - dmin + 1, [dmin](const DfgNode& x) { return x.depth - dmin; });
  pass(max_phase_ + 1, [](const DfgNode& x) { return x.phase; });
  out.order = a;
  for (size_t i = 0; i < n; ++i) {
    const DfgNode& x = nodes_[a[i]];
    if (i == 0 || x.phase != nodes_[a[i - 1]].phase || x.depth != nodes_[a[i - 1]].depth || x.op != nodes_[a[i - 1]].op) {
      if (i) out.off.push_back((int32_t)i);
      out.op.push_back(x.op);
    }
  }
  out.off.push_back((int32_t)n);
}

int dfg_build_treelstm(Dfg& g, const acrobat_trees& tr, int32_t vocab, int32_t op_leaf, int32_t op_internal,
                       std::string& err) {
  if (tr.n_trees < 0 || (tr.n_trees > 0 && !tr.tree_off)) { err = "null structure array"; return ACROBAT_EINVAL; }
  // (a batch of empty trees has no nodes and needs no child arrays, as for schedule_trees)
  if (tr.n_trees > 0 && tr.tree_off[tr.n_trees] > 0 && (!tr.left || !tr.right)) { err = "null structure array"; return ACROBAT_EINVAL; }
  struct Frame { int32_t node; int32_t stage; int32_t dl, nl; };  // local node, children done, left depth / node id
  std::vector<Frame> stack;
  for (int32_t t = 0; t < tr.n_trees; ++t) {
    const int32_t base = tr.tree_off[t], cnt = tr.tree_off[t + 1] - base;
    if (cnt < 0) { err = "tree_off not non-decreasing"; return ACROBAT_ESTRUCT; }
    if (cnt == 0) continue;
    // the root is the one node that is nobody's child
    std::vector<uint8_t> is_child((size_t)cnt, 0);
    for (int32_t j = 0; j < cnt; ++j) {
      const int32_t l = tr.left[base + j], r = tr.right[base + j];
      if ((l < 0) != (r < 0)) { err = "node with exactly one child"; return ACROBAT_ESTRUCT; }
      if (l < 0) continue;
      if (l >= cnt || r >= cnt || l == r || l == j || r == j || is_child[l] || is_child[r]) { err = "bad child index"; return ACROBAT_ESTRUCT; }
      is_child[l] = is_child[r] = 1;
    }
    int32_t root = -1;
    for (int32_t j = 0; j < cnt; ++j)
      if (!is_child[j]) {
        if (root >= 0) { err = "more than one root"; return ACROBAT_ESTRUCT; }
        root = j;
      }
    if (root < 0) { err = "no root"; return ACROBAT_ESTRUCT; }
    // the unbatched program: state, depth = eval(node)
    int32_t ret_depth = 0, ret_node = -1, visited = 0;
    stack.assign(1, Frame{root, 0, 0, -1});
    while (!stack.empty()) {
      Frame& f = stack.back();
      const int32_t gnode = base + f.node;
      const int32_t l = tr.left[gnode], r = tr.right[gnode];
      if (l < 0) {  // leaf: hoisted input transform, depth 0
        const int32_t tok = tr.token ? tr.token[gnode] : 0;
        if (vocab >= 0 && (tok < 0 || tok >= vocab)) { err = "token out of range"; return ACROBAT_ESTRUCT; }
        const int rc = g.invoke(op_leaf, 0, 0, gnode, tok, 0, -1, -1, &ret_node, err);
        if (rc != ACROBAT_OK) return rc;
        ret_depth = 0;
        ++visited;
        stack.pop_back();
        continue;
      }
      if (f.stage == 0) { f.stage = 1; stack.push_back(Frame{l, 0, 0, -1}); continue; }
      if (f.stage == 1) { f.stage = 2; f.dl = ret_depth; f.nl = ret_node; stack.push_back(Frame{r, 0, 0, -1}); continue; }
      const int32_t depth = 1 + std::max(f.dl, ret_depth);  // inline depth computation
      const int32_t nl = f.nl, nr = ret_node;
      const int rc = g.invoke(op_internal, 0, depth, gnode, base + l, base + r, nl, nr, &ret_node, err);
      if (rc != ACROBAT_OK) return rc;
      ret_depth = depth;
      ++visited;
      stack.pop_back();
      if ((int32_t)stack.size() > cnt) { err = "cycle"; return ACROBAT_ESTRUCT; }
    }
    if (visited != cnt) { err = "nodes unreachable from the root"; return ACROBAT_ESTRUCT; }
  }
  return ACROBAT_OK;
}

}  // namespace acrobat
