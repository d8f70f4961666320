"""Pins for the TreeLSTM oracle: hand-computed trees, closed forms, a library LSTM cell,
evaluation-order and batch-order invariance.  CPU only."""
import math

import numpy as np
import pytest
import torch

import oracle
from workloads import generators as gen


def tiny(left, right, token, emb, W_leaf, U, b_leaf=None, b=None, H=1, tree_off=None):
    left = np.asarray(left, np.int32)
    N = left.shape[0]
    D = np.asarray(emb).shape[1]
    return dict(n_trees=1 if tree_off is None else len(tree_off) - 1,
                tree_off=np.asarray([0, N] if tree_off is None else tree_off, np.int32),
                left=left, right=np.asarray(right, np.int32), token=np.asarray(token, np.int32),
                H=H, D=D, emb=np.asarray(emb, np.float32),
                W_leaf=np.asarray(W_leaf, np.float32).reshape(5 * H, D),
                b_leaf=np.zeros(5 * H, np.float32) if b_leaf is None else np.asarray(b_leaf, np.float32),
                U=np.asarray(U, np.float32).reshape(5 * H, 2 * H),
                b=np.zeros(5 * H, np.float32) if b is None else np.asarray(b, np.float32))


def test_single_leaf_hand_value(golden):
    g = golden("hand_cases.txt")
    for x, sign in ((1.0, 1.0), (-1.0, -1.0)):
        w = tiny([-1], [-1], [0], [[x]], [0, 7, -3, 0, 1], np.zeros(10))
        h, c = oracle.treelstm(w)
        assert c[0, 0] == pytest.approx(sign * g["tl_leaf_pos_c"], abs=1e-15)
        assert h[0, 0] == pytest.approx(sign * g["tl_leaf_pos_h"], abs=1e-15)


def test_three_node_symmetric_hand_value(golden):
    g = golden("hand_cases.txt")
    U = [[1, 1], [0, 0], [0, 0], [0, 0], [1, -1]]
    # ids: 0 = left leaf (x=+1), 1 = right leaf (x=-1), 2 = root
    w = tiny([-1, -1, 0], [-1, -1, 1], [0, 1, -1], [[1.0], [-1.0]], [0, 7, -3, 0, 1], U)
    h, c = oracle.treelstm(w)
    assert c[2, 0] == pytest.approx(g["tl_sym_root_c"], abs=1e-15)
    assert h[2, 0] == pytest.approx(g["tl_sym_root_h"], abs=1e-15)


@pytest.mark.parametrize("ids", [(0, 1, 2), (2, 0, 1), (1, 2, 0)])
def test_three_node_asymmetric_hand_value(golden, ids):
    """Root/leaf numbering must not matter; left/right and gate order must."""
    g = golden("hand_cases.txt")
    U = [[0.5, -0.5], [1, 0], [0, 1], [0.25, 0.25], [1, 1]]
    b = [0, 1, -1, 0, 0]
    L, R, root = ids
    left, right, token = [-1] * 3, [-1] * 3, [-1] * 3
    left[root], right[root] = L, R
    token[L], token[R] = 0, 1
    w = tiny(left, right, token, [[1.0], [0.5]], [1, 0, 0, -1, 2], U, b=b)
    h, c = oracle.treelstm(w)
    assert h[L, 0] == pytest.approx(g["tl_asym_left_h"], abs=1e-15)
    assert c[L, 0] == pytest.approx(g["tl_asym_left_c"], abs=1e-15)
    assert h[R, 0] == pytest.approx(g["tl_asym_right_h"], abs=1e-15)
    assert c[R, 0] == pytest.approx(g["tl_asym_right_c"], abs=1e-15)
    assert c[root, 0] == pytest.approx(g["tl_asym_root_c"], abs=1e-15)
    assert h[root, 0] == pytest.approx(g["tl_asym_root_h"], abs=1e-15)
    # exchange the children
    w["left"][root], w["right"][root] = R, L
    h, c = oracle.treelstm(w)
    assert c[root, 0] == pytest.approx(g["tl_swap_root_c"], abs=1e-15)
    assert h[root, 0] == pytest.approx(g["tl_swap_root_h"], abs=1e-15)


def test_all_zero_weights_give_zero_states():
    w = gen.treelstm_workload(3, 2, 9, 8, 17, "uniform", seed=5)
    for k in ("W_leaf", "U", "b_leaf", "b"):
        w[k] = np.zeros_like(w[k])
    h, c = oracle.treelstm(w)
    assert np.all(h == 0.0) and np.all(c == 0.0)


def test_bias_only_complete_tree_closed_form():
    """U = 0 and W_leaf = 0: c at height k of a complete tree is a geometric sum.

    c_0 = s(bl_i) tanh(bl_u);  c_k = alpha + beta c_{k-1},
    alpha = s(b_i) tanh(b_u), beta = s(b_fl) + s(b_fr)
    =>  c_k = alpha (1 - beta^k)/(1 - beta) + beta^k c_0.
    """
    H, depth = 3, 5
    n_leaves = 2 ** depth
    # complete tree: heap numbering turned into (left,right) arrays; node 0 = root
    n = 2 * n_leaves - 1
    left = np.array([2 * i + 1 if 2 * i + 1 < n else -1 for i in range(n)], np.int32)
    right = np.array([2 * i + 2 if 2 * i + 2 < n else -1 for i in range(n)], np.int32)
    token = np.where(left < 0, 0, -1).astype(np.int32)
    rng = np.random.default_rng(0)
    bl = rng.uniform(-1, 1, 5 * H).astype(np.float32)
    b = rng.uniform(-1, 1, 5 * H).astype(np.float32)
    w = tiny(left, right, token, np.ones((1, 2)), np.zeros((5 * H, 2)), np.zeros((5 * H, 2 * H)),
             b_leaf=bl, b=b, H=H)
    h, c = oracle.treelstm(w)
    s = lambda t: 1.0 / (1.0 + math.exp(-t))
    for q in range(H):
        c0 = s(bl[q]) * math.tanh(bl[4 * H + q])
        alpha = s(b[q]) * math.tanh(b[4 * H + q])
        beta = s(b[H + q]) + s(b[2 * H + q])
        for node in range(n):
            k = depth - int(math.floor(math.log2(node + 1)))  # height above the leaves
            want_c = alpha * (1 - beta ** k) / (1 - beta) + beta ** k * c0
            assert c[node, q] == pytest.approx(want_c, rel=1e-12, abs=1e-13)
            o = s(b[3 * H + q]) if k > 0 else s(bl[3 * H + q])
            assert h[node, q] == pytest.approx(o * math.tanh(want_c), rel=1e-12, abs=1e-13)


def _torch_cell(H, D, W_ih, W_hh, b_ih):
    cell = torch.nn.LSTMCell(D, H, bias=True, dtype=torch.float64)
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(W_ih))
        cell.weight_hh.copy_(torch.from_numpy(W_hh))
        cell.bias_ih.copy_(torch.from_numpy(b_ih))
        cell.bias_hh.zero_()
    return cell


def test_leaf_equals_library_lstm_cell_from_zero_state():
    """A leaf is an LSTM cell started from the zero state (its forget path multiplies 0)."""
    w = gen.treelstm_workload(2, 4, 6, 16, 23, "uniform", seed=11, bias_scale=0.5)
    H, D = w["H"], w["D"]
    h, c = oracle.treelstm(w)
    rows = lambda M, g: M[g * H:(g + 1) * H]
    # library gate order (i, f, g, o); ours (i, f_l, f_r, o, u)
    W_ih = np.concatenate([rows(w["W_leaf"], 0), rows(w["W_leaf"], 1), rows(w["W_leaf"], 4),
                           rows(w["W_leaf"], 3)]).astype(np.float64)
    b_ih = np.concatenate([rows(w["b_leaf"], 0), rows(w["b_leaf"], 1), rows(w["b_leaf"], 4),
                           rows(w["b_leaf"], 3)]).astype(np.float64)
    cell = _torch_cell(H, D, W_ih, np.zeros((4 * H, H)), b_ih)
    leaves = np.nonzero(w["left"] < 0)[0]
    x = torch.from_numpy(w["emb"][w["token"][leaves]].astype(np.float64))
    with torch.no_grad():
        th, tc = cell(x)
    np.testing.assert_allclose(h[leaves], th.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(c[leaves], tc.numpy(), rtol=1e-12, atol=1e-14)


def test_left_chain_equals_library_lstm_over_the_leaf_states():
    """Left-leaning chain with the right forget gate shut (bias -> -inf side):
    node_t = LSTMCell(input = h(right leaf_t), state = left child's (h, c)) with
    W_hh = U[:, :H] (left columns), W_ih = U[:, H:] (right columns)."""
    H, L = 8, 7
    rng = gen.make_rng(3)
    # chain: leaves 0..L-1, internal L+t has left = previous internal (or leaf 0), right = leaf t+1
    n = 2 * L - 1
    left = np.full(n, -1, np.int32)
    right = np.full(n, -1, np.int32)
    for t in range(L - 1):
        left[L + t] = 0 if t == 0 else L + t - 1
        right[L + t] = t + 1
    token = np.where(left < 0, np.arange(n), -1).astype(np.int32)
    w = tiny(left, right, token, gen.normal_f32((L, H), rng), gen.uniform_f32((5 * H, H), 0.4, rng),
             gen.uniform_f32((5 * H, 2 * H), 0.4, rng), b_leaf=gen.uniform_f32((5 * H,), 0.3, rng),
             b=gen.uniform_f32((5 * H,), 0.3, rng), H=H)
    w["b"][2 * H:3 * H] = -1000.0  # s(-1000 + O(1)) == 0 exactly in double
    h, c = oracle.treelstm(w)
    rows = lambda M, g: M[g * H:(g + 1) * H]
    pick = lambda M: np.concatenate([rows(M, 0), rows(M, 1), rows(M, 4), rows(M, 3)]).astype(np.float64)
    cell = _torch_cell(H, H, pick(w["U"][:, H:]), pick(w["U"][:, :H]), pick(w["b"]))
    th = torch.from_numpy(h[0:1].copy())
    tc = torch.from_numpy(c[0:1].copy())
    with torch.no_grad():
        for t in range(L - 1):
            x = torch.from_numpy(h[t + 1:t + 2].copy())
            th, tc = cell(x, (th, tc))
            np.testing.assert_allclose(h[L + t], th.numpy()[0], rtol=1e-12, atol=1e-14)
            np.testing.assert_allclose(c[L + t], tc.numpy()[0], rtol=1e-12, atol=1e-14)


def test_right_chain_uses_right_forget_gate():
    """Mirror image: shut the LEFT forget gate; state flows through the right child."""
    H, L = 4, 5
    rng = gen.make_rng(4)
    n = 2 * L - 1
    left = np.full(n, -1, np.int32)
    right = np.full(n, -1, np.int32)
    for t in range(L - 1):
        right[L + t] = 0 if t == 0 else L + t - 1
        left[L + t] = t + 1
    token = np.where(left < 0, np.arange(n), -1).astype(np.int32)
    w = tiny(left, right, token, gen.normal_f32((L, H), rng), gen.uniform_f32((5 * H, H), 0.4, rng),
             gen.uniform_f32((5 * H, 2 * H), 0.4, rng), b=gen.uniform_f32((5 * H,), 0.3, rng), H=H)
    w["b"][1 * H:2 * H] = -1000.0
    h, c = oracle.treelstm(w)
    rows = lambda M, g: M[g * H:(g + 1) * H]
    pick = lambda M: np.concatenate([rows(M, 0), rows(M, 2), rows(M, 4), rows(M, 3)]).astype(np.float64)
    cell = _torch_cell(H, H, pick(w["U"][:, :H]), pick(w["U"][:, H:]), pick(w["b"]))
    th, tc = torch.from_numpy(h[0:1].copy()), torch.from_numpy(c[0:1].copy())
    with torch.no_grad():
        for t in range(L - 1):
            th, tc = cell(torch.from_numpy(h[t + 1:t + 2].copy()), (th, tc))
            np.testing.assert_allclose(h[L + t], th.numpy()[0], rtol=1e-12, atol=1e-14)
            np.testing.assert_allclose(c[L + t], tc.numpy()[0], rtol=1e-12, atol=1e-14)


@pytest.fixture(scope="module")
def small_batch():
    return gen.treelstm_workload(9, 1, 14, 24, 50, "zipf1.1", seed=77, bias_scale=0.2)


def test_recursive_equals_topological_bit_for_bit(small_batch):
    h0, c0 = oracle.treelstm(small_batch)
    h1, c1 = oracle.treelstm(small_batch, topo=True)
    assert not np.isnan(h0).any() and not np.isnan(c0).any()
    assert np.array_equal(h0, h1) and np.array_equal(c0, c1)


def test_threads_do_not_change_results(small_batch):
    h0, c0 = oracle.treelstm(small_batch)
    h1, c1 = oracle.treelstm(small_batch, nthreads=4)
    assert np.array_equal(h0, h1) and np.array_equal(c0, c1)


def test_tree_order_in_batch_does_not_change_any_node(small_batch):
    w = small_batch
    h0, c0 = oracle.treelstm(w)
    order = gen.make_rng(1).permutation(w["n_trees"])
    w2, src = gen.reorder_trees(w, order, per_node={"token": w["token"]})
    h1, c1 = oracle.treelstm(w2)
    assert np.array_equal(h1, h0[src]) and np.array_equal(c1, c0[src])


def test_node_numbering_does_not_change_any_node(small_batch):
    w = small_batch
    h0, c0 = oracle.treelstm(w)
    w2, perm = gen.relabel_trees(w, gen.make_rng(2), extra={"token": w["token"]})
    h1, c1 = oracle.treelstm(w2)
    assert np.array_equal(h1[perm], h0) and np.array_equal(c1[perm], c0)


def test_single_tree_alone_equals_same_tree_in_batch(small_batch):
    w = small_batch
    h0, c0 = oracle.treelstm(w)
    t = 4
    b, e = int(w["tree_off"][t]), int(w["tree_off"][t + 1])
    w1 = dict(w)
    w1.update(n_trees=1, tree_off=np.array([0, e - b], np.int32), left=w["left"][b:e],
              right=w["right"][b:e], token=w["token"][b:e])
    h1, c1 = oracle.treelstm(w1)
    assert np.array_equal(h1, h0[b:e]) and np.array_equal(c1, c0[b:e])


def test_state_bounds(small_batch):
    w = small_batch
    h, c = oracle.treelstm(w)
    assert np.all(np.abs(h) < 1.0)
    off = w["tree_off"]
    for t in range(w["n_trees"]):
        b = int(off[t])
        for g in range(b, int(off[t + 1])):
            if w["left"][g] >= 0:
                bound = 1.0 + np.abs(c[b + w["left"][g]]) + np.abs(c[b + w["right"][g]])
                assert np.all(np.abs(c[g]) <= bound)
            else:
                assert np.all(np.abs(c[g]) <= 1.0)


def test_matches_plain_numpy_matmul_on_random_batch(small_batch):
    """Library matmul as the contraction step, Python loop over a schedule-free post-order."""
    w = small_batch
    H = w["H"]
    h0, c0 = oracle.treelstm(w)
    sg = lambda t: 1.0 / (1.0 + np.exp(-t))
    Wl, U = w["W_leaf"].astype(np.float64), w["U"].astype(np.float64)
    h = np.zeros_like(h0)
    c = np.zeros_like(c0)
    done = np.zeros(h.shape[0], bool)
    off = w["tree_off"]
    for t in range(w["n_trees"]):
        b, e = int(off[t]), int(off[t + 1])
        while not done[b:e].all():
            for g in range(b, e):
                if done[g]:
                    continue
                l, r = w["left"][g], w["right"][g]
                if l < 0:
                    z = Wl @ w["emb"][w["token"][g]].astype(np.float64) + w["b_leaf"]
                    cl = cr = 0.0
                elif done[b + l] and done[b + r]:
                    z = U @ np.concatenate([h[b + l], h[b + r]]) + w["b"]
                    cl, cr = c[b + l], c[b + r]
                else:
                    continue
                i, fl, fr, o = (sg(z[k * H:(k + 1) * H]) for k in range(4))
                u = np.tanh(z[4 * H:])
                c[g] = i * u + fl * cl + fr * cr
                h[g] = o * np.tanh(c[g])
                done[g] = True
    np.testing.assert_allclose(h0, h, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(c0, c, rtol=1e-11, atol=1e-13)
