"""Seeded synthetic inputs for the batched-dataflow-graph hot path.

This module only *draws* inputs: tree shapes, sequence lengths, token ids,
embedding tables and weights.  It contains none of the method's arithmetic
(no cell, no schedule) so that both the CPU oracle's tests and the GPU
path's tests can consume exactly the same arrays without sharing any logic.

The paper evaluates TreeLSTM and MV-RNN on parse trees of a sentiment
treebank and its recurrent models on a cross-lingual inference corpus, with
hidden sizes 256/512 (64/128 for MV-RNN), batch sizes 8/64 and untrained
parameters (paper Evaluation, "Experimental Setup" and table 3).  Neither corpus is available
here, so the generators below produce stand-ins with the same structure:
binary trees with sentence-length leaf counts, Zipf-distributed token ids,
variable-length sequences, random weights.

Conventions
-----------
* All random draws come from ``numpy.random.Generator(Philox(seed))``.
* Draw order per workload: sizes -> shapes -> token ids -> tables -> weights.
* A tree with L leaves has 2L-1 nodes.  Leaves are numbered 0..L-1 left to
  right, internal nodes follow in post-order, so the root is node 2L-2.
  ``left``/``right`` hold tree-local child ids, -1/-1 for a leaf.
* Span splitting: a span of n >= 2 leaves is split at k uniform in
  {1..n-1}; the left child takes the first k leaves.  Draws are made in
  pre-order (parent, then left subtree, then right subtree).
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 0xAC20B470


def make_rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(int(seed)))


# --------------------------------------------------------------------------
# structures
# --------------------------------------------------------------------------
def random_binary_tree(n_leaves: int, rng: np.random.Generator):
    """Return (left, right) int32 arrays of a random binary tree (see module doc)."""
    if n_leaves < 1:
        raise ValueError("a tree needs at least one leaf")
    n_nodes = 2 * n_leaves - 1
    left = np.full(n_nodes, -1, dtype=np.int32)
    right = np.full(n_nodes, -1, dtype=np.int32)
    next_internal = [n_leaves]

    def build(lo: int, hi: int) -> int:
        # span [lo, hi) of leaves -> id of the subtree root
        n = hi - lo
        if n == 1:
            return lo
        k = int(rng.integers(1, n))  # 1..n-1
        l_id = build(lo, lo + k)
        r_id = build(lo + k, hi)
        me = next_internal[0]
        next_internal[0] += 1
        left[me] = l_id
        right[me] = r_id
        return me

    root = build(0, n_leaves)
    assert root == n_nodes - 1
    return left, right


def tree_batch(leaf_counts, rng: np.random.Generator):
    """Concatenate random trees.  Returns dict(n_trees, tree_off, left, right, n_leaves)."""
    lefts, rights, off = [], [], [0]
    for L in leaf_counts:
        l, r = random_binary_tree(int(L), rng)
        lefts.append(l)
        rights.append(r)
        off.append(off[-1] + l.shape[0])
    cat = lambda xs: (np.concatenate(xs) if xs else np.zeros(0, np.int32)).astype(np.int32)
    return dict(
        n_trees=len(lefts),
        tree_off=np.asarray(off, dtype=np.int32),
        left=cat(lefts),
        right=cat(rights),
        leaf_counts=np.asarray(list(leaf_counts), dtype=np.int32),
    )


def relabel_trees(trees: dict, rng: np.random.Generator, extra: dict | None = None):
    """Randomly renumber the nodes inside every tree (structure unchanged).

    Returns (new_trees, perm) where perm[g_old] = g_new over global node ids.
    Per-node arrays in ``extra`` (e.g. token) are permuted consistently and
    returned inside new_trees.
    """
    off = trees["tree_off"]
    N = int(off[-1])
    perm = np.empty(N, dtype=np.int64)
    left = np.empty(N, dtype=np.int32)
    right = np.empty(N, dtype=np.int32)
    for t in range(trees["n_trees"]):
        b, e = int(off[t]), int(off[t + 1])
        p = rng.permutation(e - b)  # old local -> new local
        perm[b:e] = b + p
        ol, orr = trees["left"][b:e], trees["right"][b:e]
        nl = np.where(ol >= 0, p[np.maximum(ol, 0)], -1)
        nr = np.where(orr >= 0, p[np.maximum(orr, 0)], -1)
        left[b + p] = nl
        right[b + p] = nr
    out = dict(trees)
    out["left"], out["right"] = left, right
    for k, v in (extra or {}).items():
        nv = np.empty_like(v)
        nv[perm] = v
        out[k] = nv
    return out, perm


def reorder_trees(trees: dict, order, per_node: dict | None = None):
    """Put whole trees in a different order inside the batch.

    Returns (new_trees, src) with src[g_new] = g_old so that outputs of the
    reordered batch can be compared row by row: out_new[g] <-> out_old[src[g]].
    """
    off = trees["tree_off"]
    segs, new_off = [], [0]
    for t in order:
        b, e = int(off[t]), int(off[t + 1])
        segs.append(np.arange(b, e))
        new_off.append(new_off[-1] + (e - b))
    src = np.concatenate(segs) if segs else np.zeros(0, np.int64)
    out = dict(trees)
    out["tree_off"] = np.asarray(new_off, dtype=np.int32)
    out["left"] = trees["left"][src]
    out["right"] = trees["right"][src]
    if "leaf_counts" in trees:
        out["leaf_counts"] = trees["leaf_counts"][list(order)]
    for k, v in (per_node or {}).items():
        out[k] = v[src]
    return out, src


def zipf_tokens(n: int, vocab: int, exponent: float, rng: np.random.Generator):
    """n ids in [0, vocab) with P(id = k-1) proportional to k**-exponent (finite Zipf)."""
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-float(exponent))
    cdf = np.cumsum(w / w.sum())
    cdf[-1] = 1.0
    u = rng.random(n)
    return np.minimum(np.searchsorted(cdf, u, side="right"), vocab - 1).astype(np.int32)


def uniform_f32(shape, bound: float, rng: np.random.Generator):
    return rng.uniform(-bound, bound, size=shape).astype(np.float32)


def normal_f32(shape, rng: np.random.Generator):
    return rng.standard_normal(size=shape).astype(np.float32)


def leaf_mask(trees: dict):
    return trees["left"] < 0


# --------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------
def treelstm_workload(n_trees, leaf_lo, leaf_hi, H, V, token_dist, seed, bias_scale=0.0, D=None):
    """Binary TreeLSTM batch: trees, leaf token ids, embedding table and weights.

    Gate order of the 5H weight rows: (i, f_l, f_r, o, u).  U columns 0..H-1 act
    on the left child's h, H..2H-1 on the right child's.
    """
    rng = make_rng(seed)
    D = H if D is None else D  # embedding width (the benchmark configs use D == H)
    counts = rng.integers(leaf_lo, leaf_hi + 1, size=n_trees)
    trees = tree_batch(counts, rng)
    N = int(trees["tree_off"][-1])
    is_leaf = leaf_mask(trees)
    n_leaf = int(is_leaf.sum())
    if token_dist == "uniform":
        tok = rng.integers(0, V, size=n_leaf).astype(np.int32)
    elif token_dist == "zipf1.1":
        tok = zipf_tokens(n_leaf, V, 1.1, rng)
    else:
        raise ValueError(token_dist)
    token = np.full(N, -1, dtype=np.int32)
    token[is_leaf] = tok
    emb = normal_f32((V, D), rng)
    bound = 1.0 / np.sqrt(H)
    W_leaf = uniform_f32((5 * H, D), bound, rng)
    U = uniform_f32((5 * H, 2 * H), bound, rng)
    if bias_scale > 0.0:
        b_leaf = uniform_f32((5 * H,), bias_scale, rng)
        b = uniform_f32((5 * H,), bias_scale, rng)
    else:
        b_leaf = np.zeros(5 * H, np.float32)
        b = np.zeros(5 * H, np.float32)
    out = dict(trees)
    out.update(kind="treelstm", H=H, D=D, V=V, token=token, emb=emb, W_leaf=W_leaf,
               b_leaf=b_leaf, U=U, b=b, seed=seed, n_nodes=N)
    return out


def mvrnn_workload(n_trees, leaf_lo, leaf_hi, d, seed):
    """MV-RNN batch: every leaf owns one table row (token = leaf ordinal in the batch)."""
    rng = make_rng(seed)
    counts = rng.integers(leaf_lo, leaf_hi + 1, size=n_trees)
    trees = tree_batch(counts, rng)
    N = int(trees["tree_off"][-1])
    is_leaf = leaf_mask(trees)
    V = int(is_leaf.sum())
    token = np.full(N, -1, dtype=np.int32)
    token[is_leaf] = np.arange(V, dtype=np.int32)
    vec_tab = normal_f32((V, d), rng)
    mat_tab = (np.eye(d, dtype=np.float32)[None, :, :]
               + np.float32(0.01) * normal_f32((V, d, d), rng)).astype(np.float32)
    bound = 1.0 / 8.0 if d == 64 else 1.0 / np.sqrt(d)
    W = uniform_f32((d, 2 * d), bound, rng)
    WM = uniform_f32((d, 2 * d), bound, rng)
    out = dict(trees)
    out.update(kind="mvrnn", d=d, V=V, token=token, vec_tab=vec_tab, mat_tab=mat_tab,
               W=W, WM=WM, seed=seed, n_nodes=N)
    return out


def lstm_workload(n_seq, len_lo, len_hi, H, D, seed, bias_scale=0.0):
    """Variable-length LSTM batch.  Rows of x are packed sequence-major:
    row(s, t) = seq_off[s] + t.  Gate order of the 4H rows: (i, f, o, u)."""
    rng = make_rng(seed)
    lens = rng.integers(len_lo, len_hi + 1, size=n_seq).astype(np.int32)
    seq_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    total = int(seq_off[-1])
    x = normal_f32((total, D), rng)
    bound = 1.0 / np.sqrt(H)
    Wx = uniform_f32((4 * H, D), bound, rng)
    Wh = uniform_f32((4 * H, H), bound, rng)
    b = uniform_f32((4 * H,), bias_scale, rng) if bias_scale > 0 else np.zeros(4 * H, np.float32)
    return dict(kind="lstm", n_seq=n_seq, len=lens, seq_off=seq_off, H=H, D=D, x=x,
                Wx=Wx, Wh=Wh, b=b, seed=seed, n_nodes=total)


def birnn_workload(n_seq, len_lo, len_hi, H, D, n_out, seed, bias_scale=0.1):
    """Bidirectional RNN batch with a per-token output layer.  Rows of x are packed
    sequence-major (row(s, t) = seq_off[s] + t).  Each direction has its own Wx [H,D], Wh [H,H],
    b [H] and initial state [H]; the output layer is C [n_out, 2H] (columns 0..H-1 act on the
    forward state), cb [n_out]."""
    rng = make_rng(seed)
    lens = rng.integers(len_lo, len_hi + 1, size=n_seq).astype(np.int32)
    seq_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    total = int(seq_off[-1])
    out = dict(kind="birnn", n_seq=n_seq, len=lens, seq_off=seq_off, H=H, D=D, n_out=n_out, seed=seed,
               n_nodes=total, x=normal_f32((total, D), rng))
    bound = 1.0 / np.sqrt(H)
    for p in ("f", "b"):
        out[p + "Wx"] = uniform_f32((H, D), bound, rng)
        out[p + "Wh"] = uniform_f32((H, H), bound, rng)
        out[p + "b"] = uniform_f32((H,), bias_scale, rng)
        out[p + "init"] = uniform_f32((H,), 1.0, rng) * np.float32(0.5) + np.float32(0.5)
    out["C"] = uniform_f32((n_out, 2 * H), 1.0 / np.sqrt(2 * H), rng)
    out["cb"] = uniform_f32((n_out,), bias_scale, rng)
    return out


def drnn_workload(n_inst, H, n_labels, n_out, seed, max_depth=6, max_children=4, p_child=0.7, p_sibling=0.6,
                  bias_scale=0.1, cap=None, from_scores=False, topology_bias=(0.0, 0.0), weight_gain=8.0, score_gain=4.0):
    """Doubly-recurrent-network batch: one input vector per instance, from which a tree is
    generated top-down.  Parameters: label embeddings emb [n_labels, H]; ancestral, fraternal and
    predictive cells Wa, Wf, Wp [H, 2H] with biases [H]; score layer Wo [n_out, H], bo [n_out].
    The decisions (children, next sibling, label) are emulated pseudo-randomly from
    seed_decisions; max_depth levels at most, max_children children per node at most.  `cap`
    bounds the number of nodes the outputs can hold.  from_scores: the decisions are read off the
    scores instead (children iff y[0] > 0, sibling iff y[1] > 0, label = argmax of the rest); the
    two topology scores then get the biases topology_bias, which set how bushy the trees are, and the
    cell weights and the score layer are scaled up (weight_gain, score_gain): with the small weights of
    the other workloads an untrained network's scores hardly differ from node to node and every node
    would decide alike.  Whether a seed grows interesting trees is luck; users check the result."""
    rng = make_rng(seed)
    bound = 1.0 / np.sqrt(2 * H)
    out = dict(kind="drnn", n_inst=n_inst, H=H, n_labels=n_labels, n_out=n_out, seed=seed,
               seed_decisions=(int(seed) * 0x9E3779B1 + 12345) % (1 << 63), max_depth=max_depth, max_children=max_children,
               p_child=p_child, p_sibling=p_sibling, x0=uniform_f32((n_inst, H), 1.0, rng) * np.float32(0.5) + np.float32(0.5),
               emb=normal_f32((n_labels, H), rng))
    for p in ("a", "f", "p"):
        out["W" + p] = uniform_f32((H, 2 * H), bound, rng)
        out["b" + p] = uniform_f32((H,), bias_scale, rng)
    out["Wo"] = uniform_f32((n_out, H), 1.0 / np.sqrt(H), rng)
    out["bo"] = uniform_f32((n_out,), bias_scale, rng)
    out["from_scores"] = bool(from_scores)
    if from_scores:
        for p in ("a", "f", "p"):
            out["W" + p] = (out["W" + p] * np.float32(weight_gain)).astype(np.float32)
        out["Wo"] = (out["Wo"] * np.float32(score_gain)).astype(np.float32)
        # centre the topology scores (states are sigmoids, mean about 0.5) and shift them by the biases
        for r in (0, 1):
            out["bo"][r] = np.float32(topology_bias[r]) - np.float32(0.5) * out["Wo"][r].sum(dtype=np.float32)
    if cap is None:  # every instance at its largest: a full tree of max_children-ary branching
        per = sum(max_children ** d for d in range(max_depth))
        cap = min(n_inst * per, n_inst * 4096)
    out["cap"] = int(cap)
    return out


def tree_paths(t):
    """(instance, child indices from the root) of every node of a generated forest."""
    out = []
    for i in range(len(t["inst"])):
        p, j = [], i
        while t["parent"][j] >= 0:
            p.append(int(t["sib_index"][j]))
            j = int(t["parent"][j])
        out.append((int(t["inst"][i]), tuple(reversed(p))))
    return out


def match_trees(got, want):
    """Checks that two forests hold the same positions with the same label, depth and relatives;
    returns, for every node of `got`, the index of the node of `want` at the same position."""
    pg, pw = tree_paths(got), tree_paths(want)
    assert len(set(pg)) == len(pg) == len(pw) and set(pg) == set(pw), "different sets of tree positions"
    at = {p: i for i, p in enumerate(pw)}
    for i, p in enumerate(pg):
        j = at[p]
        assert got["label"][i] == want["label"][j] and got["depth"][i] == want["depth"][j]
        assert got["sib_index"][i] == want["sib_index"][j]
        for rel in ("parent", "prev"):
            a, b = int(got[rel][i]), int(want[rel][j])
            assert (a < 0) == (b < 0) and (a < 0 or pg[a] == pw[b])
    return np.array([at[p] for p in pg], np.int64)


def paper_grid_workload(model: str, size: str, batch: int, seed: int | None = None):
    """Mini-batches shaped like the paper's evaluation grid (Evaluation, "Experimental Setup"): model size small /
    large (hidden 256 / 512; MV-RNN 64 / 128) and batch size 8 / 64.  The treebank and the
    sentence-pair corpus themselves are not available: sentence lengths are drawn uniformly from
    [5, 35] (mean 20), trees are random binary splits; parameters are random, as in the paper.
    The BiRNN's output layer has 16 units.  The tree generator (no dataset in the paper either: random
    input vectors) has 30 labels, 2 + 30 scores per node, and grows trees of at most 6 levels and 4
    children per node (about 25 nodes on average, a few above 100)."""
    assert size in ("small", "large") and model in ("treelstm", "mvrnn", "birnn", "drnn")
    s = (SEED_BASE + 100 + {"treelstm": 0, "mvrnn": 10, "birnn": 20, "drnn": 30}[model] + (0 if size == "small" else 5) + batch
         if seed is None else seed)
    if model == "treelstm":
        w = treelstm_workload(batch, 5, 35, 256 if size == "small" else 512, 20000, "zipf1.1", s)
    elif model == "birnn":
        H = 256 if size == "small" else 512
        w = birnn_workload(batch, 5, 35, H, H, 16, s)
    elif model == "drnn":
        w = drnn_workload(batch, 256 if size == "small" else 512, 30, 32, s)
    else:
        w = mvrnn_workload(batch, 5, 35, 64 if size == "small" else 128, s)
    w["name"] = f"paper_{model}_{size}_bs{batch}"
    return w


# The five benchmark configurations (index = position in the baseline's list).
CONFIG_NAMES = (
    "treelstm_h256_8x20",
    "treelstm_h256_64",
    "treelstm_h512_256",
    "mvrnn_d64_64",
    "lstm_h512_256",
)


def make_config(idx: int, seed: int | None = None, n_instances: int | None = None):
    """Build benchmark configuration ``idx`` (0..4).  n_instances: the same recipe with another number of
    trees / sequences (scaling runs; the benchmark configurations proper use the default)."""
    s = SEED_BASE + idx if seed is None else seed
    n = (8, 64, 256, 64, 256)[idx] if n_instances is None else int(n_instances)
    if idx == 0:
        w = treelstm_workload(n, 20, 20, 256, 1000, "uniform", s)
    elif idx == 1:
        w = treelstm_workload(n, 10, 50, 256, 20000, "zipf1.1", s)
    elif idx == 2:
        w = treelstm_workload(n, 10, 60, 512, 20000, "zipf1.1", s)
    elif idx == 3:
        w = mvrnn_workload(n, 10, 40, 64, s)
    elif idx == 4:
        w = lstm_workload(n, 1, 100, 512, 512, s)
    else:
        raise IndexError(idx)
    w["name"] = CONFIG_NAMES[idx] if n_instances is None else f"{CONFIG_NAMES[idx]}_x{n}"
    return w
