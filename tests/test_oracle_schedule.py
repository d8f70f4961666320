"""Pins for the schedule oracle: brute force over all small binary trees, invariants."""
import itertools

import numpy as np
import pytest

import oracle
from workloads import generators as gen


def all_shapes(n_leaves):
    """Every binary tree shape with n_leaves leaves, as nested tuples (None = leaf)."""
    if n_leaves == 1:
        return [None]
    out = []
    for k in range(1, n_leaves):
        for l, r in itertools.product(all_shapes(k), all_shapes(n_leaves - k)):
            out.append((l, r))
    return out


def flatten(shape):
    """nested tuples -> (left, right) with pre-order numbering (root = 0)."""
    left, right = [], []

    def rec(s):
        me = len(left)
        left.append(-1)
        right.append(-1)
        if s is not None:
            left[me] = rec(s[0])
            right[me] = rec(s[1])
        return me

    rec(shape)
    return np.asarray(left, np.int32), np.asarray(right, np.int32)


def longest_path_by_matrix_powers(left, right):
    """depth(n) = largest k with a k-edge downward walk from n (adjacency-matrix powers)."""
    n = len(left)
    A = np.zeros((n, n), np.int64)
    for i in range(n):
        if left[i] >= 0:
            A[i, left[i]] = 1
            A[i, right[i]] = 1
    depth = np.zeros(n, np.int64)
    P = np.eye(n, dtype=np.int64)
    for k in range(1, n + 1):
        P = (P @ A > 0).astype(np.int64)
        depth[P.sum(axis=1) > 0] = k
    return depth


def test_catalan_count():
    assert [len(all_shapes(n)) for n in range(1, 7)] == [1, 1, 2, 5, 14, 42]


@pytest.mark.parametrize("n_leaves", range(1, 7))
def test_depth_is_longest_downward_path_on_every_small_tree(n_leaves):
    rng = gen.make_rng(100 + n_leaves)
    shapes = all_shapes(n_leaves)
    lefts, rights, off = [], [], [0]
    for s in shapes:
        l, r = flatten(s)
        lefts.append(l)
        rights.append(r)
        off.append(off[-1] + len(l))
    trees = dict(n_trees=len(shapes), tree_off=np.asarray(off, np.int32),
                 left=np.concatenate(lefts), right=np.concatenate(rights))
    trees, _ = gen.relabel_trees(trees, rng)
    n_levels, depth = oracle.tree_depths(trees)
    for t in range(trees["n_trees"]):
        b, e = off[t], off[t + 1]
        want = longest_path_by_matrix_powers(trees["left"][b:e], trees["right"][b:e])
        assert np.array_equal(depth[b:e], want)
    assert n_levels == depth.max() + 1


def check_tree_schedule(trees, level_off, level_nodes, lrow, rrow):
    N = int(trees["tree_off"][-1])
    # a partition of all nodes
    assert level_off[0] == 0 and level_off[-1] == N
    assert np.array_equal(np.sort(level_nodes), np.arange(N))
    level_of = np.empty(N, np.int64)
    for d in range(len(level_off) - 1):
        seg = level_nodes[level_off[d]:level_off[d + 1]]
        assert len(seg) > 0
        assert np.all(np.diff(seg) > 0)  # ascending ids inside a level
        level_of[seg] = d
    base = np.repeat(trees["tree_off"][:-1], np.diff(trees["tree_off"]))
    for p, g in enumerate(level_nodes):
        if trees["left"][g] < 0:
            assert level_of[g] == 0 and lrow[p] == -1 and rrow[p] == -1  # all leaves hoisted to level 0
        else:
            gl, gr = base[g] + trees["left"][g], base[g] + trees["right"][g]
            assert lrow[p] == gl and rrow[p] == gr
            # dependences respected, and as early as possible
            assert level_of[g] == 1 + max(level_of[gl], level_of[gr])


def test_schedule_invariants_random_batch():
    rng = gen.make_rng(9)
    trees = gen.tree_batch(rng.integers(1, 30, size=40), rng)
    trees, _ = gen.relabel_trees(trees, rng)
    check_tree_schedule(trees, *oracle.tree_schedule(trees))


def test_schedule_config0_shape():
    w = gen.make_config(0)
    level_off, level_nodes, _, _ = oracle.tree_schedule(w)
    sizes = np.diff(level_off)
    assert sizes[0] == 8 * 20 and sizes.sum() == 8 * 39 and sizes[-1] >= 1
    assert len(sizes) >= 6  # a 20-leaf binary tree is at least ceil(log2 20)=5 high


def test_sequence_schedule():
    lens = np.array([3, 0, 5, 1, 5, 2], np.int32)
    level_off, rows = oracle.seq_schedule(lens)
    off = np.concatenate([[0], np.cumsum(lens)])
    sizes = np.diff(level_off)
    assert list(sizes) == [5, 4, 3, 2, 2]
    assert sizes.sum() == lens.sum() and np.all(np.diff(sizes) <= 0)
    for t in range(5):
        want = [off[s] + t for s in range(len(lens)) if lens[s] > t]
        assert list(rows[level_off[t]:level_off[t + 1]]) == want
    # one sequence of length T: T levels of one step each (the listing's recurrence)
    level_off, rows = oracle.seq_schedule(np.array([7], np.int32))
    assert list(np.diff(level_off)) == [1] * 7 and list(rows) == list(range(7))
    level_off, rows = oracle.seq_schedule(np.zeros(0, np.int32))
    assert list(level_off) == [0] and rows.size == 0
