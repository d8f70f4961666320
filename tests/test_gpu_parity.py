"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Schedules bit exact; fp32 states within 1e-4 abs and 1e-3 per-node relative."""
import numpy as np
import pytest

import oracle
from workloads import generators as gen
from workloads import make_config

pytestmark = pytest.mark.gpu

NT = oracle.default_threads()


@pytest.fixture(scope="module")
def ctx():
    import paper_2305_10611_amd as A
    c = A.Context(0)
    yield c
    c.close()


@pytest.fixture(scope="module")
def P():
    from tests import parity
    return parity


def check_tree_schedule(ctx, w):
    level_off, level_nodes = ctx.acrobat_last_schedule()
    o_off, o_nodes, _, _ = oracle.tree_schedule(w)
    assert np.array_equal(level_off, o_off) and np.array_equal(level_nodes, o_nodes)


# ---------------------------------------------------------------- TreeLSTM
@pytest.mark.parametrize("cfg", [0, 1, 2])
def test_treelstm_benchmark_configs(ctx, P, cfg):
    w = make_config(cfg)
    h, c = P.run_treelstm(ctx, w)
    check_tree_schedule(ctx, w)
    oh, oc = oracle.treelstm(w, nthreads=NT)
    eh = P.assert_close(h, oh, f"cfg{cfg} h")
    ec = P.assert_close(c, oc, f"cfg{cfg} c")
    print(f"cfg{cfg}: N={w['n_nodes']} h abs/rel {eh[0]:.2e}/{eh[1]:.2e}  c abs/rel {ec[0]:.2e}/{ec[1]:.2e}")


@pytest.mark.parametrize("H,n_trees,lo,hi", [(32, 5, 1, 9), (64, 37, 1, 33), (96, 3, 50, 70), (256, 130, 1, 12),
                                             (512, 9, 1, 40)])
def test_treelstm_ragged_shapes_with_bias(ctx, P, H, n_trees, lo, hi):
    w = gen.treelstm_workload(n_trees, lo, hi, H, 101, "zipf1.1", seed=H + n_trees, bias_scale=0.3)
    h, c = P.run_treelstm(ctx, w)
    check_tree_schedule(ctx, w)
    oh, oc = oracle.treelstm(w, nthreads=NT)
    P.assert_close(h, oh, "h")
    P.assert_close(c, oc, "c")


def test_treelstm_embedding_width_differs_from_hidden_size(ctx, P):
    for H, D in ((64, 160), (128, 32)):
        w = gen.treelstm_workload(12, 1, 25, H, 90, "zipf1.1", seed=H + D, bias_scale=0.3, D=D)
        assert w["emb"].shape[1] == D and w["W_leaf"].shape == (5 * H, D)
        h, c = P.run_treelstm(ctx, w)
        oh, oc = oracle.treelstm(w, nthreads=NT)
        P.assert_close(h, oh, "h")
        P.assert_close(c, oc, "c")


def test_treelstm_many_tiles_per_level(ctx, P):
    """A wide, shallow batch: tens of thousands of nodes per level, several dispatch rounds."""
    w = gen.treelstm_workload(9000, 2, 6, 64, 500, "zipf1.1", seed=77, bias_scale=0.2)
    assert w["n_nodes"] > 60000
    h, c = P.run_treelstm(ctx, w)
    check_tree_schedule(ctx, w)
    oh, oc = oracle.treelstm(w, nthreads=NT)
    P.assert_close(h, oh, "h")
    P.assert_close(c, oc, "c")


def test_treelstm_null_bias_equals_zero_bias(ctx, P):
    w = gen.treelstm_workload(6, 2, 20, 64, 50, "uniform", seed=8)
    h0, c0 = P.run_treelstm(ctx, w, use_bias=True)
    h1, c1 = P.run_treelstm(ctx, w, use_bias=False)
    assert np.array_equal(h0, h1) and np.array_equal(c0, c1)


def test_treelstm_random_node_numbering(ctx, P):
    w = gen.treelstm_workload(20, 1, 30, 64, 77, "uniform", seed=9, bias_scale=0.2)
    w2, perm = gen.relabel_trees(w, gen.make_rng(10), extra={"token": w["token"]})
    h, c = P.run_treelstm(ctx, w2)
    check_tree_schedule(ctx, w2)
    oh, oc = oracle.treelstm(w2, nthreads=NT)
    P.assert_close(h, oh, "h")
    P.assert_close(c, oc, "c")
    # and the relabelled batch gives the original batch's states, row for row
    h0, c0 = P.run_treelstm(ctx, w)
    P.assert_close(h[perm], h0.astype(np.float64), "h vs original numbering")


def test_treelstm_tree_order_invariance(ctx, P):
    w = make_config(1)
    h0, c0 = P.run_treelstm(ctx, w)
    order = gen.make_rng(3).permutation(w["n_trees"])
    w2, src = gen.reorder_trees(w, order, per_node={"token": w["token"]})
    h1, c1 = P.run_treelstm(ctx, w2)
    P.assert_close(h1, h0[src].astype(np.float64), "h")
    P.assert_close(c1, c0[src].astype(np.float64), "c")
    print("bitwise equal under tree reordering:", np.array_equal(h1, h0[src]) and np.array_equal(c1, c0[src]))


def test_treelstm_degenerate_batches(ctx, P):
    import paper_2305_10611_amd as A
    # empty batch: OK, nothing launched
    w = gen.treelstm_workload(2, 1, 1, 32, 10, "uniform", seed=1)
    empty = dict(w, n_trees=0, tree_off=np.array([0], np.int32), left=np.zeros(0, np.int32),
                 right=np.zeros(0, np.int32), token=np.zeros(0, np.int32))
    h, c = P.run_treelstm(ctx, empty)
    assert h.shape[0] == 0
    # only single-leaf trees: one level
    h, c = P.run_treelstm(ctx, w)
    oh, oc = oracle.treelstm(w)
    P.assert_close(h, oh, "h")
    level_off, _ = ctx.acrobat_last_schedule()
    assert list(level_off) == [0, 2]
    # malformed structure is refused and nothing is written
    bad = dict(w, left=np.array([0, -1], np.int32))
    hh, cc = P.nan_filled(2, 32), P.nan_filled(2, 32)
    t = {k: P.dev(w[k]) for k in ("emb", "W_leaf", "U")}
    rc = ctx.acrobat_treelstm_forward(bad, 32, 32, 10, t["emb"], t["W_leaf"], None, t["U"], None, hh, cc, 0)
    assert rc == A.ESTRUCT and ctx.acrobat_last_error() != ""
    assert bool(hh.isnan().all())
    rc = ctx.acrobat_treelstm_forward(w, 33, 32, 10, t["emb"], t["W_leaf"], None, t["U"], None, hh, cc, 0)
    assert rc == A.EINVAL
    rc = ctx.acrobat_treelstm_forward(w, 32, 32, 10, None, t["W_leaf"], None, t["U"], None, hh, cc, 0)
    assert rc == A.EINVAL


def test_treelstm_deep_chain(ctx, P):
    """Many tiny levels in a row (launch-order dependence between consecutive levels)."""
    H, L = 64, 150
    rng = gen.make_rng(12)
    n = 2 * L - 1
    left = np.full(n, -1, np.int32)
    right = np.full(n, -1, np.int32)
    for t in range(L - 1):
        left[L + t] = 0 if t == 0 else L + t - 1
        right[L + t] = t + 1
    w = gen.treelstm_workload(1, 1, 1, H, 40, "uniform", seed=13, bias_scale=0.2)
    token = np.where(left < 0, rng.integers(0, 40, n), -1).astype(np.int32)
    w.update(n_trees=1, tree_off=np.array([0, n], np.int32), left=left, right=right, token=token, n_nodes=n)
    h, c = P.run_treelstm(ctx, w)
    oh, oc = oracle.treelstm(w)
    P.assert_close(h, oh, "h")
    P.assert_close(c, oc, "c")


# ---------------------------------------------------------------- MV-RNN
def test_mvrnn_benchmark_config(ctx, P):
    w = make_config(3)
    vec, mat = P.run_mvrnn(ctx, w, copy_leaves=1)
    check_tree_schedule(ctx, w)
    ov, om = oracle.mvrnn(w, nthreads=NT)
    ev = P.assert_close(vec, ov, "vec")
    em = P.assert_close(mat, om, "mat")
    print(f"cfg3: N={w['n_nodes']} vec abs/rel {ev[0]:.2e}/{ev[1]:.2e} mat abs/rel {em[0]:.2e}/{em[1]:.2e}")
    # without the leaf copy: internal rows identical, leaf rows untouched
    vec2, mat2 = P.run_mvrnn(ctx, w, copy_leaves=0)
    internal = w["left"] >= 0
    assert np.array_equal(vec2[internal], vec[internal]) and np.array_equal(mat2[internal], mat[internal])
    assert np.isnan(vec2[~internal]).all() and np.isnan(mat2[~internal]).all()


def test_mvrnn_small_ragged_and_relabelled(ctx, P):
    w = gen.mvrnn_workload(11, 1, 9, 64, seed=31)
    w2, perm = gen.relabel_trees(w, gen.make_rng(32), extra={"token": w["token"]})
    for ww in (w, w2):
        vec, mat = P.run_mvrnn(ctx, ww)
        check_tree_schedule(ctx, ww)
        ov, om = oracle.mvrnn(ww, nthreads=NT)
        P.assert_close(vec, ov, "vec")
        P.assert_close(mat, om, "mat")
    # shared table rows: two leaves reading the same row
    w3 = dict(w)
    w3["token"] = np.where(w["token"] >= 0, w["token"] % 3, -1).astype(np.int32)
    vec, mat = P.run_mvrnn(ctx, w3)
    ov, om = oracle.mvrnn(w3)
    P.assert_close(vec, ov, "vec")
    P.assert_close(mat, om, "mat")


def test_mvrnn_d128_ragged_and_relabelled(ctx, P):
    """The paper's large MV-RNN size (Evaluation, "Experimental Setup"): 128-d vectors, 128 x 128 matrices."""
    w = gen.mvrnn_workload(13, 1, 12, 128, seed=41)
    w2, perm = gen.relabel_trees(w, gen.make_rng(42), extra={"token": w["token"]})
    for ww in (w, w2):
        vec, mat = P.run_mvrnn(ctx, ww)
        check_tree_schedule(ctx, ww)
        ov, om = oracle.mvrnn(ww, nthreads=NT)
        P.assert_close(vec, ov, "vec")
        P.assert_close(mat, om, "mat")


def test_mvrnn_d128_paper_batch(ctx, P):
    from workloads.generators import paper_grid_workload
    w = paper_grid_workload("mvrnn", "large", 64)
    vec, mat = P.run_mvrnn(ctx, w, copy_leaves=0)
    ov, om = oracle.mvrnn(w, nthreads=NT)
    internal = w["left"] >= 0
    P.assert_close(vec[internal], ov[internal], "vec")
    P.assert_close(mat[internal], om[internal], "mat")
    assert np.isnan(vec[~internal]).all()


@pytest.mark.parametrize("d,trees", [(64, 40), (128, 24)])
def test_mvrnn_streaming_variant(P, d, trees):
    """Both sizes have two level kernels; the tuning hook selects the streaming one."""
    import paper_2305_10611_amd as A
    c = A.Context(0)
    try:
        assert c.acrobat_set_tuning(0, 0, 1) == A.OK
        w = gen.mvrnn_workload(trees, 1, 30, d, seed=43)
        vec, mat = P.run_mvrnn(c, w)
        ov, om = oracle.mvrnn(w, nthreads=NT)
        P.assert_close(vec, ov, "vec")
        P.assert_close(mat, om, "mat")
    finally:
        c.close()


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("trees,lo,hi,seed", [(1, 2, 2, 50), (5, 1, 9, 51), (64, 10, 40, 52), (700, 1, 12, 53), (3, 60, 90, 54)])
def test_mvrnn_all_levels_in_one_launch(ctx, P, trees, lo, hi, seed, d):
    """Every internal level in one launch, a node waiting for its own two children only (four flags per node, one
    per workgroup that writes a part of its state).  Same schedule, same tolerances; at d = 128 bit-identical to one
    launch per level (a node's arithmetic is the same code), at d = 64 equal within the tolerances (the single launch
    cuts a node's contraction into four parts instead of two).  Batches whose widest internal level exceeds 2 048
    (d = 64) or 512 (d = 128) nodes keep one launch per level."""
    import paper_2305_10611_amd as A
    w = gen.mvrnn_workload(trees, lo, hi, d, seed=seed)
    ctx.acrobat_set_profiling(True)
    try:
        vec, mat = P.run_mvrnn(ctx, w, copy_leaves=0)
        kinds = [r[0] for r in ctx.acrobat_last_profile()]
    finally:
        ctx.acrobat_set_profiling(False)
    level_off, _ = ctx.acrobat_last_schedule()
    widest = int(np.diff(level_off)[1:].max()) if len(level_off) > 2 else 0
    one_launch = len(level_off) - 1 > 2 and widest <= (2048 if d == 64 else 512)
    assert kinds == ([A.binding.K_MVRNN_PERSISTENT] if one_launch else [A.binding.K_MVRNN_LEVEL] * (len(level_off) - 2))
    assert ctx.acrobat_device_status() == A.OK
    check_tree_schedule(ctx, w)
    ov, om = oracle.mvrnn(w, nthreads=NT)
    internal = w["left"] >= 0
    P.assert_close(vec[internal], ov[internal], "vec")
    P.assert_close(mat[internal], om[internal], "mat")
    vec2, mat2 = P.run_mvrnn(ctx, w, copy_leaves=0)  # again: a new epoch, the flags of the first call are stale
    assert np.array_equal(vec2[internal], vec[internal]) and np.array_equal(mat2[internal], mat[internal])
    ctx.acrobat_set_persistent(False)
    try:
        vec1, mat1 = P.run_mvrnn(ctx, w, copy_leaves=0)
    finally:
        ctx.acrobat_set_persistent(True)
    if d == 128:
        assert np.array_equal(vec1[internal], vec[internal]) and np.array_equal(mat1[internal], mat[internal])
    else:
        P.assert_close(vec1[internal], ov[internal], "vec, one launch per level")
        P.assert_close(mat1[internal], om[internal], "mat, one launch per level")
        P.assert_close(vec[internal], vec1[internal].astype(np.float64), "vec, one launch vs one launch per level")
        P.assert_close(mat[internal], mat1[internal].astype(np.float64), "mat, one launch vs one launch per level")


@pytest.mark.parametrize("d,trees", [(64, 40), (64, 200), (128, 40)])
def test_mvrnn_persistent_wait_that_runs_out_is_reported(P, d, trees):
    """As for the recurrence: with no polls allowed, a parent whose child is not finished yet gives up, the grid
    drains, the kernel ends normally and the condition is reported once.  (d = 64: 40 trees run four workgroups per
    node, 200 trees - a widest level of more than 640 nodes - one.)"""
    import paper_2305_10611_amd as A
    w = gen.mvrnn_workload(trees, 20, 40, d, seed=55)
    c = A.Context(0)
    try:
        assert c.acrobat_set_persistent(True, 0) == A.OK
        P.run_mvrnn(c, w, copy_leaves=0)
        assert c.acrobat_device_status() == A.ETIMEOUT
        assert c.acrobat_device_status() == A.OK
        assert c.acrobat_set_persistent(True, -1) == A.OK
        vec, mat = P.run_mvrnn(c, w, copy_leaves=0)
        assert c.acrobat_device_status() == A.OK
        ov, om = oracle.mvrnn(w, nthreads=NT)
        internal = w["left"] >= 0
        P.assert_close(vec[internal], ov[internal], "vec")
        P.assert_close(mat[internal], om[internal], "mat")
    finally:
        c.close()


def test_mvrnn_rejects_unsupported_d(ctx, P):
    import paper_2305_10611_amd as A
    w = gen.mvrnn_workload(2, 2, 3, 32, seed=33)
    t = {k: P.dev(w[k]) for k in ("vec_tab", "mat_tab", "W", "WM")}
    N = w["n_nodes"]
    rc = ctx.acrobat_mvrnn_forward(w, 32, w["V"], t["vec_tab"], t["mat_tab"], t["W"], t["WM"],
                                   P.nan_filled(N, 32), P.nan_filled(N, 32, 32), 1, 0)
    assert rc == A.EINVAL


# ---------------------------------------------------------------- variable-length LSTM
def check_seq_schedule(ctx, lens):
    level_off, level_rows = ctx.acrobat_last_schedule()
    o_off, o_rows = oracle.seq_schedule(lens)
    assert np.array_equal(level_off, o_off) and np.array_equal(level_rows, o_rows)


def test_lstm_benchmark_config(ctx, P):
    w = make_config(4)
    h, c = P.run_lstm(ctx, w)
    check_seq_schedule(ctx, w["len"])
    oh, oc = oracle.varlen_lstm(w, nthreads=NT)
    eh = P.assert_close(h, oh, "h")
    ec = P.assert_close(c, oc, "c")
    print(f"cfg4: rows={w['n_nodes']} h abs/rel {eh[0]:.2e}/{eh[1]:.2e}  c abs/rel {ec[0]:.2e}/{ec[1]:.2e}")


@pytest.mark.parametrize("H,D,n_seq,lo,hi", [(32, 32, 3, 0, 5), (64, 96, 70, 0, 20), (256, 128, 300, 1, 7)])
def test_lstm_ragged_with_bias_and_empty_sequences(ctx, P, H, D, n_seq, lo, hi):
    w = gen.lstm_workload(n_seq, lo, hi, H, D, seed=H + D, bias_scale=0.3)
    h, c = P.run_lstm(ctx, w)
    check_seq_schedule(ctx, w["len"])
    oh, oc = oracle.varlen_lstm(w, nthreads=NT)
    P.assert_close(h, oh, "h")
    P.assert_close(c, oc, "c")


@pytest.mark.parametrize("H,D,n_seq,lo,hi", [(128, 32, 5, 1, 9), (128, 64, 33, 0, 40), (256, 128, 256, 1, 30), (256, 64, 100, 2, 2),
                                             (512, 64, 70, 0, 25), (512, 512, 256, 1, 100), (512, 32, 17, 60, 60),
                                             (512, 32, 150, 1, 40), (128, 32, 200, 0, 12)])
def test_lstm_whole_recurrence_in_one_launch(ctx, P, H, D, n_seq, lo, hi):
    """Shapes the persistent kernel takes (H in {128, 256, 512}, at most 256 live sequences): one launch for all
    time steps, same schedule, same tolerances; and against the one-launch-per-step path of the same library."""
    import paper_2305_10611_amd as A
    w = gen.lstm_workload(n_seq, lo, hi, H, D, seed=3 * H + D + n_seq, bias_scale=0.3)
    ctx.acrobat_set_profiling(True)
    try:
        h, c = P.run_lstm(ctx, w)
        kinds = [r[0] for r in ctx.acrobat_last_profile()]
    finally:
        ctx.acrobat_set_profiling(False)
    assert kinds == [A.binding.K_LSTM_INPUT, A.binding.K_LSTM_PERSISTENT]
    assert ctx.acrobat_device_status() == A.OK
    check_seq_schedule(ctx, w["len"])
    oh, oc = oracle.varlen_lstm(w, nthreads=NT)
    P.assert_close(h, oh, "h")
    P.assert_close(c, oc, "c")
    h2, c2 = P.run_lstm(ctx, w)  # again, without per-launch events: the launch before left its counters at zero
    assert np.array_equal(h, h2) and np.array_equal(c, c2)
    ctx.acrobat_set_persistent(False)
    try:
        ctx.acrobat_set_profiling(True)
        h1, c1 = P.run_lstm(ctx, w)
        kinds = [r[0] for r in ctx.acrobat_last_profile()]
    finally:
        ctx.acrobat_set_profiling(False)
        ctx.acrobat_set_persistent(True)
    assert kinds.count(A.binding.K_LSTM_STEP) == int(w["len"].max()) and A.binding.K_LSTM_PERSISTENT not in kinds
    P.assert_close(h1, oh, "h, one launch per step")
    P.assert_close(c1, oc, "c, one launch per step")
    P.assert_close(h, h1.astype(np.float64), "h, one launch vs one launch per step")


def test_lstm_more_sequences_than_one_persistent_launch_holds(ctx, P):
    """257 live sequences need seventeen node blocks of 16, one more than a launch holds: the call falls back to
    one launch per step."""
    import paper_2305_10611_amd as A
    w = gen.lstm_workload(257, 1, 6, 128, 32, seed=71, bias_scale=0.2)
    ctx.acrobat_set_profiling(True)
    try:
        h, c = P.run_lstm(ctx, w)
        kinds = [r[0] for r in ctx.acrobat_last_profile()]
    finally:
        ctx.acrobat_set_profiling(False)
    assert A.binding.K_LSTM_PERSISTENT not in kinds and A.binding.K_LSTM_STEP in kinds
    oh, oc = oracle.varlen_lstm(w, nthreads=NT)
    P.assert_close(h, oh, "h")
    P.assert_close(c, oc, "c")


def test_lstm_persistent_wait_that_runs_out_ends_the_kernel_and_is_reported(P):
    """The bound of the waits inside the persistent kernel, forced from the host: with no polls allowed the
    first workgroup that finds its block's previous step incomplete gives up, every workgroup leaves at its
    next poll, the kernel ends normally and acrobat_device_status reports ACROBAT_ETIMEOUT once.  The context
    then works as before."""
    import torch
    import paper_2305_10611_amd as A
    w = gen.lstm_workload(200, 30, 40, 256, 64, seed=72, bias_scale=0.2)
    c = A.Context(0)
    try:
        assert c.acrobat_set_persistent(True, 0) == A.OK
        P.run_lstm(c, w)  # synchronises
        assert c.acrobat_device_status() == A.ETIMEOUT and "gave up waiting" in c.acrobat_last_error()
        assert c.acrobat_device_status() == A.OK  # reported once
        assert c.acrobat_set_persistent(True, -1) == A.OK
        h, cc = P.run_lstm(c, w)
        assert c.acrobat_device_status() == A.OK
        oh, oc = oracle.varlen_lstm(w, nthreads=NT)
        P.assert_close(h, oh, "h")
        P.assert_close(cc, oc, "c")
    finally:
        c.close()


def test_sync_probe_reports_sane_times(ctx):
    import paper_2305_10611_amd as A
    for same_xcd, style, wt in ((1, 0, 1), (0, 0, 0), (1, 1, 0), (1, 2, 0), (0, 2, 0)):
        rc, us, phases = ctx.acrobat_sync_probe(8, 8, 200, same_xcd, style, wt, 512, 4096)
        assert rc == A.OK, ctx.acrobat_last_error()
        assert 0.2 < us < 500.0 and all(0.0 <= p < 500.0 for p in phases[:5]) and sum(phases[:5]) <= us * 1.5
    # write-once payload read with plain loads: no element may be stale, wherever the group's workgroups run
    for same_xcd in (1, 0):
        rc, us, phases = ctx.acrobat_sync_probe(8, 8, 200, same_xcd, 3, 1, 512, 4096)
        assert rc == A.OK, ctx.acrobat_last_error()
        assert phases[5] == 0.0 and 0.2 < us < 500.0
    assert ctx.acrobat_sync_probe(8, 32, 100000, 1, 3, 1, 16384, 1024)[0] == A.EINVAL  # every round's payload: over 1 GiB
    assert ctx.acrobat_sync_probe(9, 8, 10, 1, 0, 1, 512, 1024)[0] == A.EINVAL
    assert ctx.acrobat_sync_probe(1, 64, 10, 1, 2, 1, 512, 1024)[0] == A.EINVAL  # a flag line holds 32 members


def test_persistent_recurrence_after_the_probe_has_used_the_counters(ctx, P):
    """The probe leaves the arrival counters wherever its rounds took them; the next persistent launch must find
    them cleared (the recurrences otherwise leave them at zero themselves and no clearing launch runs)."""
    import paper_2305_10611_amd as A
    rc, _, _ = ctx.acrobat_sync_probe(8, 16, 37, 1, 1, 1, 256, 1024)
    assert rc == A.OK, ctx.acrobat_last_error()
    w = gen.lstm_workload(40, 1, 12, 128, 32, seed=123, bias_scale=0.2)
    for _ in range(3):  # the first call clears, the others rely on the launch before them
        h, c = P.run_lstm(ctx, w)
        assert ctx.acrobat_device_status() == A.OK
        oh, oc = oracle.varlen_lstm(w, nthreads=NT)
        P.assert_close(h, oh, "h")
        P.assert_close(c, oc, "c")
    wb = gen.birnn_workload(40, 1, 12, 128, 32, 4, seed=124, bias_scale=0.2)
    rc, _, _ = ctx.acrobat_sync_probe(8, 16, 11, 0, 1, 1, 256, 1024)
    assert rc == A.OK, ctx.acrobat_last_error()
    for _ in range(2):
        check_birnn(P, P.run_birnn(ctx, wb), oracle.birnn(wb, nthreads=NT))
        assert ctx.acrobat_device_status() == A.OK


def test_lstm_degenerate(ctx, P):
    w = gen.lstm_workload(4, 1, 3, 32, 32, seed=5)
    w0 = dict(w, len=np.zeros(4, np.int32))
    h, c = P.run_lstm(ctx, w0)
    assert h.shape[0] == 0
    w1 = dict(w, n_seq=0, len=np.zeros(0, np.int32))
    h, c = P.run_lstm(ctx, w1)
    assert h.shape[0] == 0


def test_treelstm_unfused_gather_ablation_is_bit_identical(ctx, P):
    """With gather fusion off every level first copies its operand rows into contiguous scratch; the
    level kernels then do the same arithmetic on the copies."""
    import paper_2305_10611_amd as A
    for w in (gen.treelstm_workload(40, 1, 30, 128, 300, "zipf1.1", seed=21, bias_scale=0.2, D=64), make_config(1)):
        h0, c0 = P.run_treelstm(ctx, w)
        ctx.acrobat_set_gather_fusion(False)
        try:
            h1, c1 = P.run_treelstm(ctx, w)
            ctx.acrobat_set_profiling(True)
            P.run_treelstm(ctx, w)
            rec = ctx.acrobat_last_profile()
        finally:
            ctx.acrobat_set_profiling(False)
            ctx.acrobat_set_gather_fusion(True)
        level_off, _ = ctx.acrobat_last_schedule()
        assert sum(r[0] == A.binding.K_GATHER for r in rec) == len(level_off) - 1
        assert np.array_equal(h0, h1) and np.array_equal(c0, c1)
        oh, oc = oracle.treelstm(w, nthreads=NT)
        P.assert_close(h1, oh, "h")
        P.assert_close(c1, oc, "c")


# ---------------------------------------------------------------- bidirectional RNN (program phases)
def check_birnn_schedule(ctx, lens):
    from tests.test_oracle_birnn import birnn_graph
    level_off, level_codes = ctx.acrobat_last_schedule()
    prods, R = birnn_graph(np.asarray(lens))
    if R == 0:
        assert list(level_off) == [0]
        return
    _, order, batch_off = oracle.phase_schedule(prods, np.array([0] * (2 * R) + [1] * R, np.int32))
    assert np.array_equal(level_off, batch_off) and np.array_equal(level_codes, order)


def check_birnn(P, got, want, tag=""):
    for name, g, o in zip(("hf", "hb", "y"), got, want):
        # y = relu(.) has rows that are exactly zero: their error is judged by the absolute bound only
        P.assert_close(g, o, f"{tag} {name}", ref_floor=0.1 if name == "y" else 1e-30)


@pytest.mark.parametrize("H,D,n_out,n_seq,lo,hi", [(32, 32, 1, 3, 0, 5), (64, 96, 16, 70, 0, 20), (256, 256, 16, 64, 5, 50),
                                                  (128, 64, 40, 300, 1, 7), (96, 32, 64, 33, 2, 12)])
def test_birnn_ragged_with_bias_and_empty_sequences(ctx, P, H, D, n_out, n_seq, lo, hi):
    w = gen.birnn_workload(n_seq, lo, hi, H, D, n_out, seed=H + D + n_out, bias_scale=0.3)
    got = P.run_birnn(ctx, w)
    check_birnn_schedule(ctx, w["len"])
    check_birnn(P, got, oracle.birnn(w, nthreads=NT))
    # a second call right behind the first reuses the context's index and scratch buffers
    got2 = P.run_birnn(ctx, w)
    assert all(np.array_equal(a, b) for a, b in zip(got, got2))


def test_birnn_serialised_profiling_path_and_null_bias(ctx, P):
    w = gen.birnn_workload(40, 0, 15, 64, 64, 10, seed=91, bias_scale=0.2)
    got = P.run_birnn(ctx, w)
    ctx.acrobat_set_profiling(True)
    try:
        got_serial = P.run_birnn(ctx, w)
        rec = ctx.acrobat_last_profile()
    finally:
        ctx.acrobat_set_profiling(False)
    assert all(np.array_equal(a, b) for a, b in zip(got, got_serial))
    import paper_2305_10611_amd as A
    T = int(w["len"].max())
    assert all(r[3] > 0 for r in rec)
    # one launch for both input transforms, one per step for both directions, one for the outputs
    assert sum(r[0] != A.binding.K_SPLITK_REDUCE for r in rec) == 1 + T + 1
    wz = dict(w)
    for k in ("fb", "bb", "cb"):
        wz[k] = np.zeros_like(w[k])
    g0 = P.run_birnn(ctx, wz, use_bias=True)
    g1 = P.run_birnn(ctx, wz, use_bias=False)
    assert all(np.array_equal(a, b) for a, b in zip(g0, g1))
    check_birnn(P, g1, oracle.birnn(wz, nthreads=NT))


def test_birnn_degenerate(ctx, P):
    w = gen.birnn_workload(4, 1, 3, 32, 32, 4, seed=5)
    w0 = dict(w, len=np.zeros(4, np.int32))
    hf, hb, y = P.run_birnn(ctx, w0)
    assert hf.shape[0] == 0 and y.shape[0] == 0
    w1 = gen.birnn_workload(1, 1, 1, 32, 32, 3, seed=6, bias_scale=0.5)  # one token: both directions start and end on it
    check_birnn(P, P.run_birnn(ctx, w1), oracle.birnn(w1))
    import paper_2305_10611_amd as A
    t = P.nan_filled(4, 32)
    rc = ctx.acrobat_birnn_forward(np.array([2], np.int32), 32, 32, 0, t, (t, t, None, t), (t, t, None, t), t, None, t, t, t)
    assert rc == A.EINVAL


@pytest.mark.parametrize("H,D,n_seq,lo,hi", [(128, 32, 5, 1, 9), (128, 64, 33, 0, 40), (256, 128, 256, 1, 30), (256, 64, 17, 2, 2),
                                             (512, 64, 70, 0, 25), (512, 512, 64, 5, 35), (512, 32, 16, 40, 40),
                                             (512, 64, 256, 1, 12)])
def test_birnn_both_recurrences_in_one_launch(ctx, P, H, D, n_seq, lo, hi):
    """Shapes the persistent kernel takes (H in {128, 256, 512}, at most 256 non-empty sequences): one launch
    for all steps of both directions, same schedule, same tolerances; and against one launch per step."""
    import paper_2305_10611_amd as A
    w = gen.birnn_workload(n_seq, lo, hi, H, D, 7, seed=5 * H + D + n_seq, bias_scale=0.3)
    ctx.acrobat_set_profiling(True)
    try:
        g = P.run_birnn(ctx, w)
        kinds = [r[0] for r in ctx.acrobat_last_profile() if r[0] != A.binding.K_SPLITK_REDUCE]
    finally:
        ctx.acrobat_set_profiling(False)
    assert kinds == [A.binding.K_RNN_INPUT, A.binding.K_RNN_PERSISTENT, A.binding.K_RNN_OUTPUT]
    assert ctx.acrobat_device_status() == A.OK
    ref = oracle.birnn(w, nthreads=NT)
    check_birnn(P, g, ref, "one launch")
    g2 = P.run_birnn(ctx, w)  # again, without per-launch events: the launch before left its counters at zero
    assert all(np.array_equal(a, b) for a, b in zip(g, g2))
    ctx.acrobat_set_persistent(False)
    try:
        ctx.acrobat_set_profiling(True)
        g1 = P.run_birnn(ctx, w)
        kinds = [r[0] for r in ctx.acrobat_last_profile()]
    finally:
        ctx.acrobat_set_profiling(False)
        ctx.acrobat_set_persistent(True)
    assert kinds.count(A.binding.K_RNN_STEP) == int(w["len"].max()) and A.binding.K_RNN_PERSISTENT not in kinds
    check_birnn(P, g1, ref, "one launch per step")
    for a, b, name in zip(g, g1, ("hf", "hb", "y")):
        P.assert_close(a, b.astype(np.float64), name + ", one launch vs one launch per step", ref_floor=0.1 if name == "y" else 1e-30)


def test_birnn_shapes_the_persistent_launch_does_not_take(ctx, P):
    """257 non-empty sequences need more blocks than one launch holds, H = 64 is not instantiated, and a single
    step needs no recurrence: one launch per step."""
    import paper_2305_10611_amd as A
    for n_seq, lo, hi, H in ((257, 1, 5, 128), (20, 1, 9, 64), (9, 1, 1, 128)):
        w = gen.birnn_workload(n_seq, lo, hi, H, 32, 4, seed=n_seq + H, bias_scale=0.2)
        ctx.acrobat_set_profiling(True)
        try:
            g = P.run_birnn(ctx, w)
            kinds = [r[0] for r in ctx.acrobat_last_profile()]
        finally:
            ctx.acrobat_set_profiling(False)
        assert A.binding.K_RNN_PERSISTENT not in kinds and A.binding.K_RNN_STEP in kinds
        check_birnn(P, g, oracle.birnn(w, nthreads=NT))


def test_birnn_persistent_wait_that_runs_out_ends_the_kernel_and_is_reported(P):
    """As for the LSTM: with no polls allowed a workgroup that finds its block's previous step incomplete gives
    up, the grid drains, the kernel ends normally and the status is reported once."""
    import paper_2305_10611_amd as A
    w = gen.birnn_workload(200, 20, 30, 512, 64, 5, seed=73, bias_scale=0.2)
    c = A.Context(0)
    try:
        assert c.acrobat_set_persistent(True, 0) == A.OK
        P.run_birnn(c, w)  # synchronises
        assert c.acrobat_device_status() == A.ETIMEOUT and "gave up waiting" in c.acrobat_last_error()
        assert c.acrobat_device_status() == A.OK  # reported once
        assert c.acrobat_set_persistent(True, -1) == A.OK
        g = P.run_birnn(c, w)
        assert c.acrobat_device_status() == A.OK
        check_birnn(P, g, oracle.birnn(w, nthreads=NT))
    finally:
        c.close()


# ---------------------------------------------------------------- profiling mode
def test_profiling_records_every_launch(ctx, P):
    w = make_config(0)
    ctx.acrobat_set_profiling(True)
    try:
        P.run_treelstm(ctx, w)
        rec = ctx.acrobat_last_profile()
    finally:
        ctx.acrobat_set_profiling(False)
    import paper_2305_10611_amd as A
    level_off, _ = ctx.acrobat_last_schedule()
    assert all(r[3] > 0 for r in rec)
    # a k-split level has a second record for its reduction kernel right behind it
    for prev, r in zip(rec, rec[1:]):
        if r[0] == A.binding.K_SPLITK_REDUCE:
            assert prev[0] != A.binding.K_SPLITK_REDUCE and prev[5] > 1 and prev[1:3] == r[1:3]
    assert sum(r[0] == A.binding.K_SPLITK_REDUCE for r in rec) == sum(r[5] > 1 for r in rec if r[0] != A.binding.K_SPLITK_REDUCE)
    rec = [r for r in rec if r[0] != A.binding.K_SPLITK_REDUCE]
    assert len(rec) == len(level_off) - 1
    assert [r[2] for r in rec] == list(np.diff(level_off))


# ---------------------------------------------------------------- every kernel variant
@pytest.mark.parametrize("tile,ksplit", [(64, 1), (32, 1), (64, 2), (64, 4), (32, 8), (32, 2), (6, 4), (6, 8), (65, 1), (33, 1), (16, 1)])
def test_every_tile_and_split_variant_matches_the_oracle(P, tile, ksplit):
    """The launcher normally picks the node-tile height and k split from the level size; the
    tuning hook forces one variant for every level (leaf, internal, LSTM input and steps).
    Tile 6 is the kernel for latency-bound levels (its second number is the slabs moved per step)."""
    import paper_2305_10611_amd as A
    c = A.Context(0)
    try:
        assert c.acrobat_set_tuning(tile, ksplit, 0) == A.OK
        w = gen.treelstm_workload(23, 1, 40, 256, 300, "zipf1.1", seed=tile + ksplit, bias_scale=0.2)
        h, cc = P.run_treelstm(c, w)
        oh, oc = oracle.treelstm(w, nthreads=NT)
        P.assert_close(h, oh, "h")
        P.assert_close(cc, oc, "c")
        s = gen.lstm_workload(150, 0, 9, 128, 64, seed=tile * 3 + ksplit, bias_scale=0.2)
        h, cc = P.run_lstm(c, s)
        oh, oc = oracle.varlen_lstm(s, nthreads=NT)
        P.assert_close(h, oh, "lstm h")
        P.assert_close(cc, oc, "lstm c")
        b = gen.birnn_workload(90, 0, 9, 128, 64, 20, seed=tile * 5 + ksplit, bias_scale=0.2)
        check_birnn(P, P.run_birnn(c, b), oracle.birnn(b, nthreads=NT), "birnn")
    finally:
        c.close()


@pytest.mark.parametrize("H,D", [(32, 32), (96, 160), (160, 96), (512, 64)])
def test_small_level_kernel_ragged_contraction_and_tiles(P, H, D):
    """The kernel for small levels (tile 16) deals the 16-k groups of the contraction range to four wavefronts:
    ranges of 2, 6, 10, 12 ... groups leave some wavefronts with fewer groups or none; node counts from 1 to a few
    16-node tiles with a ragged last tile; unit tiles of 3, 4, 5 or 16 units that do not divide H; an output layer
    of 5 units; both directions of a recurrence in one launch with different row counts."""
    import paper_2305_10611_amd as A
    c = A.Context(0)
    try:
        assert c.acrobat_set_tuning(16, 1, 0) == A.OK
        c.acrobat_set_profiling(True)
        w = gen.treelstm_workload(7, 1, 19, H, 60, "zipf1.1", seed=H + D, bias_scale=0.3, D=D)
        h, cc = P.run_treelstm(c, w)
        assert all(r[4] == 16 for r in c.acrobat_last_profile())
        oh, oc = oracle.treelstm(w, nthreads=NT)
        P.assert_close(h, oh, "h")
        P.assert_close(cc, oc, "c")
        c.acrobat_set_persistent(False)
        s = gen.lstm_workload(21, 0, 7, H, D, seed=H * 3 + D, bias_scale=0.2)
        h, cc = P.run_lstm(c, s)
        oh, oc = oracle.varlen_lstm(s, nthreads=NT)
        P.assert_close(h, oh, "lstm h")
        P.assert_close(cc, oc, "lstm c")
        b = gen.birnn_workload(19, 0, 6, H, D, 5, seed=H * 5 + D, bias_scale=0.2)
        check_birnn(P, P.run_birnn(c, b), oracle.birnn(b, nthreads=NT), "birnn")
    finally:
        c.close()


def test_two_contexts_on_two_streams_overlap_their_mini_batches(P):
    """Two contexts, each with a stream of its own, are handed mini-batches in turn without any synchronisation in
    between (what `bench.py` reports as two_stream_throughput): level launches of one batch overlap those of the
    other - including levels cut into equal shares, whose parked pieces and tile counters are per context - and
    every batch still matches the oracle."""
    import torch
    import paper_2305_10611_amd as A
    ws = [gen.treelstm_workload(200, 1, 40, 512, 300, "zipf1.1", seed=900 + i, bias_scale=0.2) for i in range(2)]
    refs = [oracle.treelstm(w, nthreads=NT) for w in ws]
    ctxs, streams = [A.Context(0), A.Context(0)], [torch.cuda.Stream(), torch.cuda.Stream()]
    try:
        t = [{k: P.dev(w[k]) for k in ("emb", "W_leaf", "b_leaf", "U", "b")} for w in ws]
        outs = []
        for rep in range(6):
            i = rep % 2
            w, N, H = ws[i], int(ws[i]["tree_off"][-1]), 512
            h, c = P.nan_filled(N, H), P.nan_filled(N, H)
            ctxs[i].check(ctxs[i].acrobat_treelstm_forward(w, H, int(w["D"]), int(w["V"]), t[i]["emb"], t[i]["W_leaf"], t[i]["b_leaf"],
                                                           t[i]["U"], t[i]["b"], h, c, streams[i].cuda_stream))
            outs.append((i, h, c))
        torch.cuda.synchronize()
        for i, h, c in outs:
            P.assert_close(h.cpu().numpy(), refs[i][0], "h")
            P.assert_close(c.cpu().numpy(), refs[i][1], "c")
    finally:
        for c_ in ctxs:
            c_.close()


def test_single_launch_calls_from_two_streams_take_turns(P):
    """The calls that run as one launch whose workgroups wait for each other (LSTM and BiRNN recurrences, MV-RNN
    dataflow) must not share the GPU; handed to two contexts on two streams in turn, without synchronisation, the
    library orders them itself: every result matches the oracle and no wait runs out."""
    import torch
    import paper_2305_10611_amd as A
    wl = gen.lstm_workload(256, 1, 40, 512, 64, seed=31, bias_scale=0.2)
    wm = gen.mvrnn_workload(48, 10, 30, 64, seed=32)
    wb = gen.birnn_workload(64, 5, 25, 256, 64, 8, seed=33, bias_scale=0.2)
    ref_l, ref_m, ref_b = oracle.varlen_lstm(wl, nthreads=NT), oracle.mvrnn(wm, nthreads=NT), oracle.birnn(wb, nthreads=NT)
    ctxs, streams = [A.Context(0), A.Context(0)], [torch.cuda.Stream(), torch.cuda.Stream()]
    try:
        tl = {k: P.dev(wl[k]) for k in ("x", "Wx", "Wh", "b")}
        tm = {k: P.dev(wm[k]) for k in ("vec_tab", "mat_tab", "W", "WM")}
        Rl, Nm, dm = int(wl["len"].sum()), int(wm["tree_off"][-1]), 64
        outs = []
        for rep in range(8):
            i = rep % 2
            c, st = ctxs[i], streams[i].cuda_stream
            if rep % 4 < 2:
                h, cc = P.nan_filled(Rl, 512), P.nan_filled(Rl, 512)
                c.check(c.acrobat_varlen_lstm_forward(wl["len"], 512, 64, tl["x"], tl["Wx"], tl["Wh"], tl["b"], h, cc, st))
                outs.append(("lstm", h, cc))
            else:
                vec, mat = P.nan_filled(Nm, dm), P.nan_filled(Nm, dm, dm)
                c.check(c.acrobat_mvrnn_forward(wm, dm, int(wm["V"]), tm["vec_tab"], tm["mat_tab"], tm["W"], tm["WM"], vec, mat, 0, st))
                outs.append(("mvrnn", vec, mat))
        torch.cuda.synchronize()
        assert all(c.acrobat_device_status() == A.OK for c in ctxs)
        internal = wm["left"] >= 0
        for kind, a, b in outs:
            if kind == "lstm":
                P.assert_close(a.cpu().numpy(), ref_l[0], "h")
                P.assert_close(b.cpu().numpy(), ref_l[1], "c")
            else:
                P.assert_close(a.cpu().numpy()[internal], ref_m[0][internal], "vec")
                P.assert_close(b.cpu().numpy()[internal], ref_m[1][internal], "mat")
        # (the BiRNN through the ordinary runner, on the default stream, right behind them)
        check_birnn(P, P.run_birnn(ctxs[0], wb), ref_b)
        assert ctxs[0].acrobat_device_status() == A.OK
    finally:
        for c_ in ctxs:
            c_.close()


# ---------------------------------------------------------------- stream capture
def test_forward_recorded_into_a_graph_replays_the_eager_result():
    """A captured forward call (index upload + every level launch) replayed several times, with eager work
    on another context and synchronisations between the replays, gives the eager result each time."""
    import torch
    import paper_2305_10611_amd as A
    from tests import parity as P
    w = gen.treelstm_workload(30, 1, 25, 128, 200, "zipf1.1", seed=44, bias_scale=0.2)
    other = gen.treelstm_workload(9, 1, 12, 64, 50, "uniform", seed=45)
    N, H = int(w["tree_off"][-1]), int(w["H"])
    t = {k: P.dev(w[k]) for k in ("emb", "W_leaf", "b_leaf", "U", "b")}
    ctx, ctx2 = A.Context(0), A.Context(0)
    try:
        h_ref, c_ref = P.run_treelstm(ctx, w)          # also sizes the context's buffers
        h, c = P.nan_filled(N, H), P.nan_filled(N, H)
        s = torch.cuda.Stream()
        fwd = lambda: ctx.acrobat_treelstm_forward(w, H, int(w["D"]), int(w["V"]), t["emb"], t["W_leaf"], t["b_leaf"],
                                                   t["U"], t["b"], h, c, s.cuda_stream)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s, capture_error_mode="relaxed"):
            rc = fwd()
        assert rc == A.OK, ctx.acrobat_last_error()
        assert torch.isnan(h).all()                      # capture launches nothing
        for _ in range(3):
            h.fill_(float("nan")); c.fill_(float("nan"))
            P.run_treelstm(ctx2, other)                  # eager work in between, on its own context
            g.replay()
            torch.cuda.synchronize()
            assert np.array_equal(h.cpu().numpy(), h_ref) and np.array_equal(c.cpu().numpy(), c_ref)
        # a capture that would have to allocate is refused, not attempted
        big = gen.treelstm_workload(400, 20, 40, 128, 200, "zipf1.1", seed=46)
        tb = {k: P.dev(big[k]) for k in ("emb", "W_leaf", "b_leaf", "U", "b")}
        Nb = int(big["tree_off"][-1])
        hb, cb = P.nan_filled(Nb, H), P.nan_filled(Nb, H)
        g2 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g2, stream=s, capture_error_mode="relaxed"):
            rc = ctx.acrobat_treelstm_forward(big, H, int(big["D"]), int(big["V"]), tb["emb"], tb["W_leaf"], tb["b_leaf"],
                                              tb["U"], tb["b"], hb, cb, s.cuda_stream)
        assert rc == A.EINVAL and "capture" in ctx.acrobat_last_error()
    finally:
        ctx.close(); ctx2.close()


def test_persistent_recurrences_recorded_into_a_graph_replay_the_eager_result():
    """The one-launch recurrences (LSTM, BiRNN) clear their arrival counters with a kernel, not a memset, so a
    captured call can be replayed: every replay, with eager work on another context in between, gives the eager
    result bit for bit.  (The MV-RNN dataflow launch is not captured: a captured call keeps one launch per level.)"""
    import torch
    import paper_2305_10611_amd as A
    from tests import parity as P
    w = gen.lstm_workload(40, 1, 12, 128, 64, seed=91, bias_scale=0.2)
    b = gen.birnn_workload(30, 1, 10, 128, 64, 6, seed=92, bias_scale=0.2)
    other = gen.treelstm_workload(9, 1, 12, 64, 50, "uniform", seed=45)
    ctx, ctx2 = A.Context(0), A.Context(0)
    try:
        h_ref, c_ref = P.run_lstm(ctx, w)  # also sizes the context's buffers
        R, H = int(np.sum(w["len"])), int(w["H"])
        t = {k: P.dev(w[k]) for k in ("x", "Wx", "Wh", "b")}
        h, c = P.nan_filled(R, H), P.nan_filled(R, H)
        s = torch.cuda.Stream()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s, capture_error_mode="relaxed"):
            rc = ctx.acrobat_varlen_lstm_forward(w["len"], H, int(w["D"]), t["x"], t["Wx"], t["Wh"], t["b"], h, c, s.cuda_stream)
        assert rc == A.OK, ctx.acrobat_last_error()
        for _ in range(3):
            h.fill_(float("nan")); c.fill_(float("nan"))
            P.run_treelstm(ctx2, other)
            g.replay()
            torch.cuda.synchronize()
            assert np.array_equal(h.cpu().numpy(), h_ref) and np.array_equal(c.cpu().numpy(), c_ref)
        assert ctx.acrobat_device_status() == A.OK

        ref = P.run_birnn(ctx, b)
        Rb, Hb, n_out = int(np.sum(b["len"])), int(b["H"]), int(b["n_out"])
        names = ("x", "fWx", "fWh", "fb", "finit", "bWx", "bWh", "bb", "binit", "C", "cb")
        tb = {k: P.dev(np.asarray(b[k], np.float32)) for k in names}
        hf, hb, y = P.nan_filled(Rb, Hb), P.nan_filled(Rb, Hb), P.nan_filled(Rb, n_out)
        g2 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g2, stream=s, capture_error_mode="relaxed"):
            rc = ctx.acrobat_birnn_forward(b["len"], Hb, int(b["D"]), n_out, tb["x"], (tb["fWx"], tb["fWh"], tb["fb"], tb["finit"]),
                                           (tb["bWx"], tb["bWh"], tb["bb"], tb["binit"]), tb["C"], tb["cb"], hf, hb, y, s.cuda_stream)
        assert rc == A.OK, ctx.acrobat_last_error()
        for _ in range(3):
            for o in (hf, hb, y):
                o.fill_(float("nan"))
            P.run_treelstm(ctx2, other)
            g2.replay()
            torch.cuda.synchronize()
            assert all(np.array_equal(o.cpu().numpy(), r) for o, r in zip((hf, hb, y), ref))
        assert ctx.acrobat_device_status() == A.OK
    finally:
        ctx.close(); ctx2.close()


# ---------------------------------------------------------------- generic dataflow-graph runtime
def treelstm_ops(g, B, t, w, h, c, N):
    H, D, V = int(w["H"]), int(w["D"]), int(w["V"])
    rc, leaf = g.acrobat_dfg_register_op(B.EPI_TREE_LEAF, H, nseg=1, kseg=D, src0=t["emb"], ld0=D, W=t["W_leaf"], ldw=D,
                                         bias=t["b_leaf"], h=h, c=c, src0_rows=V, out_rows=N)
    assert rc == 0
    rc, internal = g.acrobat_dfg_register_op(B.EPI_TREE_INTERNAL, H, nseg=2, kseg=H, src0=h, ld0=H, src1=h, ld1=H,
                                             W=t["U"], ldw=2 * H, bias=t["b"], h=h, c=c, cprev_src=c, src0_rows=N,
                                             src1_rows=N, out_rows=N)
    assert rc == 0
    return leaf, internal


@pytest.mark.parametrize("cfg", [0, 1])
def test_generic_runtime_treelstm_program_is_bit_identical_to_the_specialised_path(ctx, P, cfg):
    import torch
    import paper_2305_10611_amd as A
    from paper_2305_10611_amd import binding as B
    w = make_config(cfg)
    w, _ = gen.relabel_trees(w, gen.make_rng(cfg + 70), extra={"token": w["token"]})
    N, H = int(w["tree_off"][-1]), int(w["H"])
    t = {k: P.dev(w[k]) for k in ("emb", "W_leaf", "b_leaf", "U", "b")}
    h, c = P.nan_filled(N, H), P.nan_filled(N, H)
    g = A.Dfg(ctx)
    leaf, internal = treelstm_ops(g, B, t, w, h, c, N)
    assert g.acrobat_dfg_build_treelstm(w, int(w["V"]), leaf, internal) == A.OK
    oh, oc = oracle.treelstm(w, nthreads=NT)
    # The program numbers its nodes in the order it creates them, so inside a level the generic runtime lists
    # them in another order than the specialised call (ascending arena row).  Levels that are cut into equal
    # shares add a tile's pieces at share boundaries, which depend on where the tile sits in its level: both
    # paths are within tolerance of the oracle, but bit-identical only with whole tiles (forced here first).
    ctx.check(ctx.acrobat_set_tuning(64, 1, 0))
    try:
        ctx.check(g.acrobat_dfg_run(P.stream_handle()))
        torch.cuda.synchronize()
        h_ref, c_ref = P.run_treelstm(ctx, w)
        assert np.array_equal(h.cpu().numpy(), h_ref) and np.array_equal(c.cpu().numpy(), c_ref)
    finally:
        ctx.check(ctx.acrobat_set_tuning(0, 0, 0))
    h.fill_(float("nan")); c.fill_(float("nan"))
    ctx.check(g.acrobat_dfg_run(P.stream_handle()))
    torch.cuda.synchronize()
    h_ref, c_ref = h.cpu().numpy().copy(), c.cpu().numpy().copy()
    P.assert_close(h_ref, oh, "h")
    P.assert_close(c_ref, oc, "c")
    hs, cs = P.run_treelstm(ctx, w)
    P.assert_close(hs, h_ref.astype(np.float64), "specialised vs generic h")
    P.assert_close(cs, c_ref.astype(np.float64), "specialised vs generic c")
    # a second run of the same graph, and a run after clear + rebuild
    h.fill_(float("nan")); c.fill_(float("nan"))
    g.acrobat_dfg_clear()
    assert g.acrobat_dfg_build_treelstm(w, int(w["V"]), leaf, internal) == A.OK
    ctx.check(g.acrobat_dfg_run(P.stream_handle()))
    torch.cuda.synchronize()
    assert np.array_equal(h.cpu().numpy(), h_ref)
    g.close()


def test_generic_runtime_birnn_program_with_phases(ctx, P):
    """The BiRNN written node by node against invoke(): hoisted input transforms (phase 0), the two
    recurrences with inline depths (phase 1), every output operator in phase 2."""
    import torch
    import paper_2305_10611_amd as A
    from paper_2305_10611_amd import binding as B
    w = gen.birnn_workload(12, 0, 9, 64, 32, 5, seed=33, bias_scale=0.3)
    R, H, D, n_out = int(w["len"].sum()), 64, 32, 5
    names = ("x", "fWx", "fWh", "fb", "finit", "bWx", "bWh", "bb", "binit", "C", "cb")
    t = {k: P.dev(np.asarray(w[k], np.float32)) for k in names}
    hf, hb, y = P.nan_filled(R + 1, H), P.nan_filled(R + 1, H), P.nan_filled(R, n_out)
    # row R of each state arena holds the direction's initial state, so step 0 reads it like any other row
    hf[R] = t["finit"]; hb[R] = t["binit"]
    xpf, xpb = P.nan_filled(R, H), P.nan_filled(R, H)
    g = A.Dfg(ctx)
    ok = lambda r: (r[0] == A.OK and r[1]) if isinstance(r, tuple) else r
    reg = lambda *a, **k: (lambda r: (r[1] if r[0] == A.OK else pytest.fail(g.acrobat_dfg_last_error())))(g.acrobat_dfg_register_op(*a, **k))
    proj = [reg(B.EPI_STORE_Z1, H, nseg=1, kseg=D, src0=t["x"], ld0=D, W=t[p + "Wx"], ldw=D, bias=t[p + "b"], zout=z,
                src0_rows=R, out_rows=R) for p, z in (("f", xpf), ("b", xpb))]
    step = [reg(B.EPI_RNN_STEP, H, nseg=1, kseg=H, src0=hh, ld0=H, W=t[p + "Wh"], ldw=H, zadd=z, h=hh, src0_rows=R + 1,
                out_rows=R) for p, z, hh in (("f", xpf, hf), ("b", xpb, hb))]
    out = reg(B.EPI_RELU_OUT, 32, nseg=2, kseg=H, src0=hf, ld0=H, src1=hb, ld1=H, W=t["C"], ldw=2 * H, bias=t["cb"],
              n_cols=n_out, y=y, ldo=n_out, src0_rows=R, src1_rows=R, out_rows=R)
    off = w["seq_off"]
    for s in range(w["n_seq"]):
        b, T = int(off[s]), int(w["len"][s])
        pf = [g.acrobat_dfg_invoke(proj[0], 0, 0, b + i, b + i)[1] for i in range(T)]
        pb = [g.acrobat_dfg_invoke(proj[1], 0, 0, b + i, b + i)[1] for i in range(T)]
        nf, nb = [None] * T, [None] * T
        for k in range(T):  # depth k in both directions
            i = k
            rc, nf[i] = g.acrobat_dfg_invoke(step[0], 1, k, b + i, R if k == 0 else b + i - 1, 0, pf[i], -1 if k == 0 else nf[i - 1])
            assert rc == A.OK
            i = T - 1 - k
            rc, nb[i] = g.acrobat_dfg_invoke(step[1], 1, k, b + i, R if k == 0 else b + i + 1, 0, pb[i], -1 if k == 0 else nb[i + 1])
            assert rc == A.OK
        for i in range(T):
            assert g.acrobat_dfg_invoke(out, 2, 0, b + i, b + i, b + i, nf[i], nb[i])[0] == A.OK
    boff, order, bops = g.acrobat_dfg_schedule()
    T_max = int(w["len"].max())
    assert len(bops) == 2 + 2 * T_max + 1 and boff[-1] - boff[-2] == R
    ctx.check(g.acrobat_dfg_run(P.stream_handle()))
    torch.cuda.synchronize()
    ohf, ohb, oy = oracle.birnn(w, nthreads=NT)
    P.assert_close(hf[:R].cpu().numpy(), ohf, "hf")
    P.assert_close(hb[:R].cpu().numpy(), ohb, "hb")
    P.assert_close(y.cpu().numpy(), oy, "y", ref_floor=0.1)
    g.close()


# ---------------------------------------------------------------- large batches, sampled parity
def test_treelstm_large_batch_sampled_against_the_oracle(ctx, P):
    """4096 trees (about 290 000 nodes, leaf level of about 147 000): every kernel variant at grid sizes far
    beyond the benchmark configurations.  Trees are independent, so the oracle evaluates a sample of them."""
    w = gen.treelstm_workload(4096, 10, 60, 256, 20000, "zipf1.1", seed=501, bias_scale=0.1)
    h, c = P.run_treelstm(ctx, w)
    assert not np.isnan(h).any() and not np.isnan(c).any()
    check_tree_schedule(ctx, w)
    off = w["tree_off"]
    for first in (0, 2048, 4096 - 48):
        b, e = int(off[first]), int(off[first + 48])
        sub = dict(w, n_trees=48, tree_off=(off[first:first + 49] - off[first]).astype(np.int32), left=w["left"][b:e],
                   right=w["right"][b:e], token=w["token"][b:e])
        oh, oc = oracle.treelstm(sub, nthreads=NT)
        P.assert_close(h[b:e], oh, f"h of trees {first}..")
        P.assert_close(c[b:e], oc, f"c of trees {first}..")


def test_lstm_many_sequences_sampled_against_the_oracle(ctx, P):
    w = gen.lstm_workload(3000, 0, 60, 256, 128, seed=502, bias_scale=0.1)
    h, c = P.run_lstm(ctx, w)
    assert not np.isnan(h).any()
    check_seq_schedule(ctx, w["len"])
    off = np.concatenate([[0], np.cumsum(w["len"])])
    for first in (0, 1500, 3000 - 40):
        b, e = int(off[first]), int(off[first + 40])
        sub = dict(w, n_seq=40, len=w["len"][first:first + 40], x=w["x"][b:e])
        oh, oc = oracle.varlen_lstm(sub, nthreads=NT)
        P.assert_close(h[b:e], oh, f"h of sequences {first}..")
        P.assert_close(c[b:e], oc, f"c of sequences {first}..")


DRNN_KINDS = {4: "cell", 6: "scores"}


def check_drnn(P, w, trees, states, want):
    at = P.match_trees(trees, want)
    for name, got in zip(("a", "f", "g", "y"), states):
        assert got.shape[0] == len(at)
        P.assert_close(got, want[name][at], "drnn " + name)


@pytest.mark.parametrize("mode", (0, 1, 2))
@pytest.mark.parametrize("ghosts", (False, True))
def test_drnn_matches_the_oracle_in_every_mode(ctx, P, mode, ghosts):
    """Tensor-dependent control flow (section 4.2): the same trees and states whether nodes are
    evaluated one by one, one per instance at a time, or with every subtree on its own fiber."""
    w = gen.drnn_workload(11, 64, 9, 32, seed=91, max_depth=5, max_children=4, bias_scale=0.3)
    want = oracle.drnn(w)
    rc, trees, st, states = P.run_drnn(ctx, w, mode, ghosts)
    assert st["n_nodes"] == len(want["inst"]) and st["n_ghosts"] == (int((trees["sib_index"] > 0).sum()) if ghosts else 0)
    check_drnn(P, w, trees, states, want)
    # the host-only run of the program takes the same decisions, in the same evaluations
    import paper_2305_10611_amd as A
    rc2, trees2, st2 = A.acrobat_drnn_schedule(w, mode, ghosts)
    assert rc2 == A.OK and st2 == st
    for k in trees:
        assert np.array_equal(trees[k], trees2[k])


def test_drnn_paper_batch_without_bias_and_profile(ctx, P):
    from workloads.generators import paper_grid_workload
    w = paper_grid_workload("drnn", "small", 64)
    want = oracle.drnn(w)
    n = len(want["inst"])
    ctx.acrobat_set_profiling(True)
    try:
        rc, trees, st, states = P.run_drnn(ctx, w)
        recs = ctx.acrobat_last_profile()
    finally:
        ctx.acrobat_set_profiling(False)
    check_drnn(P, w, trees, states, want)
    assert st["n_rounds"] == trees["round"].max() + 1
    assert all(r[0] == 12 and r[3] > 0 for r in recs)  # generic-runtime batches, each with a measured time
    # rows: every node passes through the ancestral, fraternal and predictive cell and the score layer
    assert sum(r[2] for r in recs) == 4 * n
    # the ancestral and the later-sibling fraternal batch of an evaluation share one launch
    assert len(recs) < st["n_buckets"]
    w0 = dict(w, ba=np.zeros_like(w["ba"]), bf=np.zeros_like(w["bf"]), bp=np.zeros_like(w["bp"]), bo=np.zeros_like(w["bo"]))
    rc, trees0, st0, states0 = P.run_drnn(ctx, w, use_bias=False)
    check_drnn(P, w0, trees0, states0, oracle.drnn(w0))


def test_drnn_large_hidden_size_and_wide_levels(ctx, P):
    w = gen.drnn_workload(48, 512, 16, 32, seed=92, max_depth=5, max_children=4)
    want = oracle.drnn(w)
    rc, trees, st, states = P.run_drnn(ctx, w)
    check_drnn(P, w, trees, states, want)


def test_drnn_degenerate_and_error_cases(ctx, P):
    import paper_2305_10611_amd as A
    w = gen.drnn_workload(6, 64, 3, 32, seed=93)
    want = oracle.drnn(w)
    n = len(want["inst"])
    rc, trees, st, states = P.run_drnn(ctx, w, max_nodes=n)  # exactly enough room
    check_drnn(P, w, trees, states, want)
    rc, trees, st, _ = P.run_drnn(ctx, w, max_nodes=n - 1, check=False)
    assert rc == A.ENOMEM and "max_nodes" in ctx.acrobat_last_error() and st["n_nodes"] == n - 1
    rc, trees, st, states = P.run_drnn(ctx, dict(w, n_inst=0, x0=w["x0"][:0]), check=False)
    assert rc == A.OK and st["n_nodes"] == 0
    rc, trees, st, _ = P.run_drnn(ctx, w, max_nodes=0, check=False)  # no room at all
    assert rc == A.ENOMEM and st["n_nodes"] == 0
    w1 = dict(w, max_depth=1)  # roots only: one evaluation
    rc, trees, st, states = P.run_drnn(ctx, w1)
    assert st["n_nodes"] == 6 and st["n_rounds"] == 1
    check_drnn(P, w1, trees, states, oracle.drnn(w1))
    for bad in (dict(w, max_children=0), dict(w, p_sibling=-0.5), dict(w, max_depth=0)):
        assert P.run_drnn(ctx, bad, check=False)[0] == A.EINVAL
    # sizes the kernels do not take are refused before anything is touched
    t = {k: P.dev(np.asarray(w[k], np.float32)) for k in ("x0", "emb", "Wa", "Wf", "Wp", "Wo")}
    buf = P.nan_filled(n, 64)
    for bad in (dict(w, H=48), dict(w, n_out=20), dict(w, n_labels=0)):
        rc, _, _ = ctx.acrobat_drnn_forward(bad, t["x0"], t, buf, buf, buf, buf, max_nodes=n)
        assert rc == A.EINVAL
    rc, _, _ = ctx.acrobat_drnn_forward(w, t["x0"], dict(t, Wp=None), buf, buf, buf, buf, max_nodes=n)
    assert rc == A.EINVAL and "null" in ctx.acrobat_last_error()


def test_ghost_operations_do_not_change_results(ctx, P):
    """Two ops in a row for half of the rows, the second op alone for the rest (a conditional): with a
    ghost on the short branch the second op runs as one batch; the values are those without it."""
    import torch
    import paper_2305_10611_amd as A
    from paper_2305_10611_amd import binding as B
    H, n = 64, 40
    rng = gen.make_rng(94)
    x = P.dev(gen.uniform_f32((n, H), 1.0, rng))
    W1, W2 = (P.dev(gen.uniform_f32((H, H), 0.125, rng)) for _ in range(2))
    outs = []
    for use_ghost in (False, True):
        h1, h2 = P.nan_filled(n, H), P.nan_filled(n, H)
        g = A.Dfg(ctx)
        rc, op1 = g.acrobat_dfg_register_op(B.EPI_RNN_STEP, H, nseg=1, kseg=H, src0=x, ld0=H, W=W1, ldw=H, h=h1, src0_rows=n, out_rows=n)
        assert rc == A.OK
        # rows that skipped op1 read x, the others read h1: two ops with the same weights
        rc, op2a = g.acrobat_dfg_register_op(B.EPI_RNN_STEP, H, nseg=1, kseg=H, src0=h1, ld0=H, W=W2, ldw=H, h=h2, src0_rows=n, out_rows=n)
        rc, op2b = g.acrobat_dfg_register_op(B.EPI_RNN_STEP, H, nseg=1, kseg=H, src0=x, ld0=H, W=W2, ldw=H, h=h2, src0_rows=n, out_rows=n)
        for i in range(n):
            if i % 2 == 0:
                rc, a = g.acrobat_dfg_invoke(op1, 0, 0, i, i)
                assert g.acrobat_dfg_invoke(op2a, 0, 1, i, i, 0, a)[0] == A.OK
            elif use_ghost:
                rc, gh = g.acrobat_dfg_ghost(0, 0)
                assert g.acrobat_dfg_invoke(op2b, 0, 1, i, i, 0, gh)[0] == A.OK
            else:
                assert g.acrobat_dfg_invoke(op2b, 0, 0, i, i)[0] == A.OK
        off, order, bops = g.acrobat_dfg_schedule()
        assert len(bops) == 3 and len(order) == n + n // 2
        ctx.check(g.acrobat_dfg_run(P.stream_handle()))
        torch.cuda.synchronize()
        outs.append(h2.cpu().numpy())
        g.close()
    assert not np.isnan(outs[0]).any() and np.array_equal(outs[0], outs[1])
    sig = lambda z: 1.0 / (1.0 + np.exp(-z))
    xd = x.cpu().numpy().astype(np.float64)
    h1d = sig(xd @ W1.cpu().numpy().astype(np.float64).T)
    src = np.where((np.arange(n) % 2 == 0)[:, None], h1d, xd)
    P.assert_close(outs[1], sig(src @ W2.cpu().numpy().astype(np.float64).T), "h2")


@pytest.mark.parametrize("mode", (1, 2))
def test_drnn_decisions_read_off_the_scores(ctx, P, mode):
    """Truly tensor-dependent control flow: whether a node has children, whether a sibling follows and
    its label are computed from the scores the score kernel stored for it.  Decisions taken from
    fp32 scores equal those from the oracle's fp64 scores as long as no score is near its threshold:
    the margins of this workload are checked first (they are thousands of times the fp32 error)."""
    w = gen.drnn_workload(24, 64, 30, 32, seed=128, from_scores=True)
    want = oracle.drnn(w)
    y = want["y"]
    top2 = np.sort(y[:, 2:], axis=1)[:, -2:]
    assert min(np.abs(y[:, 0]).min(), np.abs(y[:, 1]).min(), (top2[:, 1] - top2[:, 0]).min()) > 1e-3
    assert len(want["inst"]) > 300 and len(set(want["label"].tolist())) >= 3
    rc, trees, st, states = P.run_drnn(ctx, w, mode, True)
    assert st["n_nodes"] == len(want["inst"])
    check_drnn(P, w, trees, states, want)


@pytest.mark.parametrize("d", (64, 128))
def test_generic_runtime_mvrnn_program(ctx, P, d):
    """The matrix-vector cell as an op of the generic runtime: the recursive program invokes it once per
    internal node with the depth computed inline; leaves are read in place through their codes."""
    import torch
    import paper_2305_10611_amd as A
    from paper_2305_10611_amd import binding as B
    w = gen.mvrnn_workload(14, 1, 13, d, seed=97)
    w, _ = gen.relabel_trees(w, gen.make_rng(98), extra={"token": w["token"]})
    N, V = int(w["tree_off"][-1]), int(w["V"])
    t = {k: P.dev(w[k]) for k in ("vec_tab", "mat_tab", "W", "WM")}
    vec, mat = P.nan_filled(N, d), P.nan_filled(N, d, d)
    g = A.Dfg(ctx)
    rc, op = g.acrobat_dfg_register_op(B.EPI_MVRNN, d, src0=t["vec_tab"], src1=t["mat_tab"], W=t["W"], W2=t["WM"], h=vec, c=mat,
                                       src0_rows=V, out_rows=N)
    assert rc == A.OK, g.acrobat_dfg_last_error()
    left, right, token, off = w["left"], w["right"], w["token"], w["tree_off"]

    def evaluate(base, j):  # -> (child code, depth, producer node)
        gnode = base + j
        if left[gnode] < 0:
            return -(int(token[gnode]) + 1), 0, -1
        cl, dl, pl = evaluate(base, int(left[gnode]))
        cr, dr, pr = evaluate(base, int(right[gnode]))
        depth = 1 + max(dl, dr)
        rc, node = g.acrobat_dfg_invoke(op, 0, depth, gnode, cl, cr, pl, pr)
        assert rc == A.OK, g.acrobat_dfg_last_error()
        return gnode, depth, node

    for tr in range(w["n_trees"]):
        b, e = int(off[tr]), int(off[tr + 1])
        children = set(left[b:e][left[b:e] >= 0].tolist()) | set(right[b:e][right[b:e] >= 0].tolist())
        root = [j for j in range(e - b) if j not in children][0]
        evaluate(b, root)
    ctx.check(g.acrobat_dfg_run(P.stream_handle()))
    torch.cuda.synchronize()
    internal = left >= 0
    ov, om = oracle.mvrnn(w, nthreads=NT)
    P.assert_close(vec.cpu().numpy()[internal], ov[internal], "vec")
    P.assert_close(mat.cpu().numpy()[internal], om[internal], "mat")
    assert torch.isnan(vec[torch.from_numpy(~internal).cuda()]).all()  # leaves are read in place, never copied
    # same kernels, same batches (one per height) as the specialised entry point with one launch per level: the same bits
    ctx.acrobat_set_persistent(False)
    try:
        sv, sm = P.run_mvrnn(ctx, w, copy_leaves=0)
    finally:
        ctx.acrobat_set_persistent(True)
    assert np.array_equal(vec.cpu().numpy()[internal], sv[internal]) and np.array_equal(mat.cpu().numpy()[internal], sm[internal])
    boff, order, bops = g.acrobat_dfg_schedule()
    level_off, _ = ctx.acrobat_last_schedule()
    assert np.array_equal(np.diff(boff), np.diff(level_off)[1:])
    g.close()


def test_generic_runtime_lstm_program(ctx, P):
    """Listing 2 through invoke(): the hoisted input transform of every step at depth 0 of phase 0, step t of a
    sequence at depth t of phase 1 (the first step is an op of its own: it has no previous state)."""
    import torch
    import paper_2305_10611_amd as A
    from paper_2305_10611_amd import binding as B
    w = gen.lstm_workload(19, 0, 14, 64, 32, seed=99, bias_scale=0.2)
    R, H, D = int(w["len"].sum()), 64, 32
    t = {k: P.dev(w[k]) for k in ("x", "Wx", "Wh", "b")}
    h, c, xp = P.nan_filled(R, H), P.nan_filled(R, H), P.nan_filled(R, 4 * H)
    g = A.Dfg(ctx)

    def reg(*a, **k):
        rc, op = g.acrobat_dfg_register_op(*a, **k)
        assert rc == A.OK, g.acrobat_dfg_last_error()
        return op
    proj = reg(B.EPI_STORE_Z, H, nseg=1, kseg=D, src0=t["x"], ld0=D, W=t["Wx"], ldw=D, bias=t["b"], zout=xp, src0_rows=R, out_rows=R)
    first = reg(B.EPI_LSTM_STEP, H, zadd=xp, h=h, c=c, out_rows=R)
    step = reg(B.EPI_LSTM_STEP, H, nseg=1, kseg=H, src0=h, ld0=H, W=t["Wh"], ldw=H, zadd=xp, h=h, c=c, cprev_src=c,
               src0_rows=R, out_rows=R)
    seq_off = np.concatenate([[0], np.cumsum(w["len"])])
    for s_ in range(len(w["len"])):
        b, T = int(seq_off[s_]), int(w["len"][s_])
        prev = -1
        for i in range(T):
            rc, p = g.acrobat_dfg_invoke(proj, 0, 0, b + i, b + i)
            assert rc == A.OK
            if i == 0:
                rc, prev = g.acrobat_dfg_invoke(first, 1, 0, b, 0, 0, p)
            else:
                rc, prev = g.acrobat_dfg_invoke(step, 1, i, b + i, b + i - 1, 0, p, prev)
            assert rc == A.OK, g.acrobat_dfg_last_error()
    boff, order, bops = g.acrobat_dfg_schedule()
    T_max = int(w["len"].max())
    assert list(bops) == [proj, first] + [step] * (T_max - 1)
    assert list(np.diff(boff)[1:]) == [int((w["len"] > k).sum()) for k in range(T_max)]
    ctx.check(g.acrobat_dfg_run(P.stream_handle()))
    torch.cuda.synchronize()
    oh, oc = oracle.varlen_lstm(w)
    P.assert_close(h.cpu().numpy(), oh, "h")
    P.assert_close(c.cpu().numpy(), oc, "c")
    sh, sc = P.run_lstm(ctx, w)  # H = 64: the specialised call also takes one launch per step here
    assert np.array_equal(h.cpu().numpy(), sh) and np.array_equal(c.cpu().numpy(), sc)
    g.close()


def test_drnn_many_instances(ctx, P):
    """512 instances at once: evaluations with about a thousand nodes per batch (several node tiles, the wide
    kernels instead of the latency-bound ones), thousands of fibers alive."""
    w = gen.drnn_workload(512, 128, 30, 32, seed=95)
    want = oracle.drnn(w)
    assert len(want["inst"]) > 10000
    rc, trees, st, states = P.run_drnn(ctx, w)
    assert st["n_fibers"] > 2000 and st["n_rounds"] < 30
    check_drnn(P, w, trees, states, want)


@pytest.mark.parametrize("H,n_inst", [(256, 256), (512, 192)])
def test_drnn_two_groups_with_every_level_split_along_k(P, H, n_inst):
    """From 192 instances on two groups of instances are in flight on two streams.  With every level forced
    to split its contraction range, both groups park partial tiles in the workspace between the two launches
    of a level at the same time: each group must have a region of its own."""
    import paper_2305_10611_amd as A
    c = A.Context(0)
    try:
        assert c.acrobat_set_tuning(64, 4, 0) == A.OK
        w = gen.drnn_workload(n_inst, H, 12, 32, seed=97 + H, max_depth=4, max_children=3, bias_scale=0.2)
        want = oracle.drnn(w)
        rc, trees, st, states = P.run_drnn(c, w, mode=A.TDC_FORK_JOIN)
        assert set(trees["inst"][trees["round"] == 0] % 2) == {0, 1}  # both groups ran
        check_drnn(P, w, trees, states, want)
    finally:
        c.close()


def test_drnn_two_groups_with_wide_batches_that_split_on_their_own(ctx, P):
    """H = 512 and 1 300 roots per group: the launcher itself splits these batches along k (no tuning hook),
    in both groups at once."""
    w = gen.drnn_workload(2600, 512, 8, 32, seed=98, max_depth=2, max_children=2, bias_scale=0.2)
    want = oracle.drnn(w)
    rc, trees, st, states = P.run_drnn(ctx, w)
    check_drnn(P, w, trees, states, want)


def test_drnn_refuses_stream_capture(ctx, P):
    """A call that must read tensor values on the host between its launches cannot be recorded into a graph."""
    import torch
    import paper_2305_10611_amd as A
    w = gen.drnn_workload(4, 64, 5, 32, seed=96)
    P.run_drnn(ctx, w)  # buffers exist already: the refusal below is not about allocation
    t = {k: P.dev(np.asarray(w[k], np.float32)) for k in ("x0", "emb", "Wa", "ba", "Wf", "bf", "Wp", "bp", "Wo", "bo")}
    cap = int(w["cap"])
    a, f, g = (P.nan_filled(cap, 64) for _ in range(3))
    y = P.nan_filled(cap, 32)
    s = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s, capture_error_mode="relaxed"):
        rc, trees, st = ctx.acrobat_drnn_forward(w, t["x0"], t, a, f, g, y, stream=s.cuda_stream)
    assert rc == A.EINVAL and "captured" in ctx.acrobat_last_error() and st["n_nodes"] == 0
    torch.cuda.synchronize()
    assert torch.isnan(a).all()
    rc, trees, st, states = P.run_drnn(ctx, w)  # and the context still works
    check_drnn(P, w, trees, states, oracle.drnn(w))


def test_saturated_gates_stay_finite(ctx, P):
    """Pre-activations of several hundred in both directions: the fast sigmoid / tanh forms must saturate to
    0, 1 and -1 without producing inf or NaN.  (With weights this large an fp32 pre-activation is only good to
    about 1e-3, so the few gates that happen to land near their transition differ from the oracle by that much:
    the comparison here is loose; the tolerances proper are tested at ordinary scales.)"""
    def loosely_close(got, want, what):
        assert np.isfinite(got).all(), what
        diff = np.abs(got.astype(np.float64) - want)
        assert diff.max() < 0.05 and (diff > 1e-3).mean() < 0.01, f"{what}: max {diff.max():.2e}, {(diff > 1e-3).mean():.2%} above 1e-3"

    w = gen.treelstm_workload(12, 1, 24, 64, 50, "uniform", seed=88, bias_scale=0.0)
    rng = gen.make_rng(89)
    for k in ("W_leaf", "U"):
        w[k] = (w[k] * np.float32(400.0)).astype(np.float32)
    w["b_leaf"] = gen.uniform_f32(w["b_leaf"].shape, 300.0, rng)
    w["b"] = gen.uniform_f32(w["b"].shape, 300.0, rng)
    h, c = P.run_treelstm(ctx, w)
    oh, oc = oracle.treelstm(w, nthreads=NT)
    assert np.abs(oc).max() > 3.0 and (np.abs(oh) > 0.999).any() and (np.abs(oh) < 1e-6).any()  # saturated both ways
    assert np.abs(h).max() <= 1.0
    loosely_close(h, oh, "h")
    loosely_close(c, oc, "c")
    s_ = gen.lstm_workload(20, 1, 12, 64, 32, seed=90, bias_scale=0.0)
    for k in ("Wx", "Wh"):
        s_[k] = (s_[k] * np.float32(400.0)).astype(np.float32)
    s_["b"] = gen.uniform_f32(s_["b"].shape, 300.0, rng)
    h, c = P.run_lstm(ctx, s_)
    oh, oc = oracle.varlen_lstm(s_, nthreads=NT)
    loosely_close(h, oh, "lstm h")
    loosely_close(c, oc, "lstm c")
    m = gen.mvrnn_workload(6, 2, 9, 64, seed=91)
    m["W"] = (m["W"] * np.float32(300.0)).astype(np.float32)  # tanh(W v) saturates
    vec, mat = P.run_mvrnn(ctx, m)
    ov, om = oracle.mvrnn(m, nthreads=NT)
    internal = m["left"] >= 0
    assert (np.abs(ov[internal]) > 0.999).any() and np.abs(vec[internal]).max() <= 1.0
    loosely_close(vec[internal], ov[internal], "vec")
