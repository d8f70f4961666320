"""Pins for the MV-RNN oracle: hand values, identities, linearity by path products."""
import numpy as np
import pytest

import oracle
from workloads import generators as gen


def mv(left, right, token, vec_tab, mat_tab, W, WM):
    left = np.asarray(left, np.int32)
    d = np.asarray(vec_tab).shape[1]
    return dict(n_trees=1, tree_off=np.asarray([0, len(left)], np.int32), left=left,
                right=np.asarray(right, np.int32), token=np.asarray(token, np.int32), d=d,
                vec_tab=np.asarray(vec_tab, np.float32), mat_tab=np.asarray(mat_tab, np.float32),
                W=np.asarray(W, np.float32).reshape(d, 2 * d), WM=np.asarray(WM, np.float32).reshape(d, 2 * d))


def test_d1_hand_value(golden):
    g = golden("hand_cases.txt")
    w = mv([-1, -1, 0], [-1, -1, 1], [0, 1, -1], [[0.5], [-0.25]], [[[1.0]], [[2.0]]],
           [0.125, -0.0625], [0.125, 0.0625])
    vec, mat = oracle.mvrnn(w)
    assert vec[2, 0] == pytest.approx(g["mv_d1_p"], abs=1e-15)
    assert mat[2, 0, 0] == pytest.approx(g["mv_d1_P"], abs=1e-15)
    assert vec[0, 0] == 0.5 and mat[1, 0, 0] == 2.0  # leaves = table rows


def test_d2_hand_value(golden):
    g = golden("hand_cases.txt")
    W = [[.125, .25, .375, .5], [-.125, -.25, -.375, -.5]]
    WM = [[.5, 0, 0, .5], [0, .5, .5, 0]]
    w = mv([-1, -1, 0], [-1, -1, 1], [0, 1, -1], [[1, 0], [0, 1]],
           [[[1, 2], [3, 4]], [[0, 1], [1, 0]]], W, WM)
    vec, mat = oracle.mvrnn(w)
    np.testing.assert_allclose(vec[2], g["mv_d2_p"], atol=1e-15)
    np.testing.assert_allclose(mat[2].ravel(), g["mv_d2_P"], atol=1e-15)
    # exchanging the children changes [B a ; A b] to [A b ; B a] and
    # P to 0.5*[[B00+A10, B01+A11],[B10+A00, B11+A01]]
    w["left"][2], w["right"][2] = 1, 0
    vec, mat = oracle.mvrnn(w)
    np.testing.assert_allclose(vec[2], g["mv_d2_swap_p"], atol=1e-15)
    np.testing.assert_allclose(mat[2], [[1.5, 2.5], [1.0, 1.0]], atol=1e-15)


def test_identity_matrices_are_a_fixed_point():
    """W_M = [I/2, I/2] and every leaf matrix = I  =>  every node matrix = I."""
    w = gen.mvrnn_workload(3, 2, 9, 4, seed=1)
    d = w["d"]
    w["mat_tab"] = np.broadcast_to(np.eye(d, dtype=np.float32), w["mat_tab"].shape).copy()
    w["WM"] = np.concatenate([np.eye(d), np.eye(d)], axis=1).astype(np.float32) * 0.5
    vec, mat = oracle.mvrnn(w)
    assert np.array_equal(mat, np.broadcast_to(np.eye(d), mat.shape))
    # and then v = [a ; b], p = tanh(W [a;b]) for nodes whose children are leaves
    off = w["tree_off"]
    for t in range(w["n_trees"]):
        b0 = int(off[t])
        for g in range(b0, int(off[t + 1])):
            l, r = w["left"][g], w["right"][g]
            if l >= 0:
                v = np.concatenate([vec[b0 + l], vec[b0 + r]])
                np.testing.assert_allclose(vec[g], np.tanh(w["W"].astype(np.float64) @ v), atol=1e-14)


def test_zero_W_gives_zero_vectors_at_internal_nodes():
    w = gen.mvrnn_workload(2, 2, 7, 4, seed=2)
    w["W"] = np.zeros_like(w["W"])
    vec, _ = oracle.mvrnn(w)
    assert np.all(vec[w["left"] >= 0] == 0.0)


def test_node_matrix_is_sum_over_leaves_of_path_products():
    """P is linear in the leaf matrices: P_node = sum_leaf (prod of W_M half-blocks on the path) A_leaf,
    the left half-block when the path descends into a left child, the right one otherwise."""
    w = gen.mvrnn_workload(4, 1, 6, 3, seed=3)
    d = w["d"]
    vec, mat = oracle.mvrnn(w)
    ML = w["WM"][:, :d].astype(np.float64)
    MR = w["WM"][:, d:].astype(np.float64)
    off = w["tree_off"]

    def leaves_with_paths(b0, g, prefix):
        l, r = w["left"][g], w["right"][g]
        if l < 0:
            yield g, prefix
        else:
            yield from leaves_with_paths(b0, b0 + l, prefix @ ML)
            yield from leaves_with_paths(b0, b0 + r, prefix @ MR)

    for t in range(w["n_trees"]):
        b0 = int(off[t])
        for g in range(b0, int(off[t + 1])):
            want = np.zeros((d, d))
            for leaf, path in leaves_with_paths(b0, g, np.eye(d)):
                want += path @ w["mat_tab"][w["token"][leaf]].astype(np.float64)
            np.testing.assert_allclose(mat[g], want, rtol=1e-12, atol=1e-13)


def test_vector_path_uses_the_other_childs_matrix():
    """One internal node, d = 3: p = tanh(W [B a ; A b]) against library matmul."""
    w = gen.mvrnn_workload(1, 2, 2, 3, seed=4)
    vec, mat = oracle.mvrnn(w)
    a, b = (w["vec_tab"][i].astype(np.float64) for i in (0, 1))
    A, B = (w["mat_tab"][i].astype(np.float64) for i in (0, 1))
    want = np.tanh(w["W"].astype(np.float64) @ np.concatenate([B @ a, A @ b]))
    np.testing.assert_allclose(vec[2], want, rtol=1e-13)
    np.testing.assert_allclose(mat[2], w["WM"].astype(np.float64) @ np.vstack([A, B]), rtol=1e-13)


def test_order_and_numbering_invariance_and_threads():
    w = gen.mvrnn_workload(7, 1, 9, 4, seed=5)
    v0, m0 = oracle.mvrnn(w)
    v1, m1 = oracle.mvrnn(w, nthreads=3)
    assert np.array_equal(v0, v1) and np.array_equal(m0, m1)
    w2, src = gen.reorder_trees(w, gen.make_rng(6).permutation(w["n_trees"]), per_node={"token": w["token"]})
    v2, m2 = oracle.mvrnn(w2)
    assert np.array_equal(v2, v0[src]) and np.array_equal(m2, m0[src])
    w3, perm = gen.relabel_trees(w, gen.make_rng(7), extra={"token": w["token"]})
    v3, m3 = oracle.mvrnn(w3)
    assert np.array_equal(v3[perm], v0) and np.array_equal(m3[perm], m0)
