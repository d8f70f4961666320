"""Tensor-dependent control flow, host side (no GPU): the tree-generation program on fibers
against the oracle's trees, the evaluation each node lands in, ghost operations."""
import numpy as np
import pytest

import oracle
import paper_2305_10611_amd as A
from paper_2305_10611_amd import binding as B
from workloads import generators as gen

MODES = (A.TDC_SEQUENTIAL, A.TDC_INSTANCE_FIBERS, A.TDC_FORK_JOIN)


def assert_same_trees(got, want):
    from tests.parity import match_trees
    return match_trees(got, want)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("ghosts", (False, True))
def test_every_mode_generates_the_oracles_trees(mode, ghosts):
    w = gen.drnn_workload(23, 32, 11, 32, seed=81, max_depth=5, max_children=4)
    want = oracle.drnn(w)
    rc, got, st = A.acrobat_drnn_schedule(w, mode, ghosts)
    assert rc == A.OK and st["n_nodes"] == len(want["inst"])
    assert_same_trees(got, want)
    n = st["n_nodes"]
    per_inst = np.bincount(want["inst"], minlength=w["n_inst"])
    if mode == A.TDC_SEQUENTIAL:  # one evaluation per node, nodes in the oracle's order
        assert st["n_rounds"] == n and st["n_fibers"] == 0
        assert list(got["round"]) == list(range(n))
        for k in ("inst", "parent", "prev", "sib_index", "depth", "label"):
            assert np.array_equal(got[k], want[k])
    elif mode == A.TDC_INSTANCE_FIBERS:  # every instance advances by one node per evaluation
        assert st["n_rounds"] == per_inst.max() and st["n_fibers"] == w["n_inst"]
        for s in range(w["n_inst"]):
            assert list(got["round"][got["inst"] == s]) == list(range(per_inst[s]))
    else:  # a node follows its parent by (index among the siblings + 1) evaluations
        for i in range(n):
            p = int(got["parent"][i])
            assert got["round"][i] == (got["round"][p] + got["sib_index"][i] + 1 if p >= 0 else 0)
        assert st["n_rounds"] == got["round"].max() + 1
        # one fiber per instance, one more per subtree that grows while its root's siblings are still generated
        has_child, has_next = np.zeros(n, bool), np.zeros(n, bool)
        has_child[got["parent"][got["parent"] >= 0]] = True
        has_next[got["prev"][got["prev"] >= 0]] = True
        assert st["n_fibers"] == w["n_inst"] + int((has_child & has_next).sum())
    assert st["n_ghosts"] == (int((got["sib_index"] > 0).sum()) if ghosts else 0)


def test_ghosts_give_one_batch_per_operator_and_evaluation():
    w = gen.drnn_workload(200, 32, 5, 32, seed=82, max_depth=5, max_children=4)
    rc, t, with_ghosts = A.acrobat_drnn_schedule(w, A.TDC_FORK_JOIN, True)
    rc2, _, without = A.acrobat_drnn_schedule(w, A.TDC_FORK_JOIN, False)
    assert rc == rc2 == A.OK and with_ghosts["n_rounds"] == without["n_rounds"]
    # From 192 instances on they are dealt out to two groups (even / odd), each evaluated on its own.  Operators present in
    # an evaluation of a group: ancestral cell (root variant in evaluation 0), fraternal cell of later siblings,
    # predictive cell, scores; the constant fraternal state of first children is computed with the group's
    # roots, and the first children's own rows are written by one batch at the very end.
    want = int((t["parent"] >= 0).any())
    for grp in (0, 1):
        mine = t["inst"] % 2 == grp
        want += 1
        for r in range(int(t["round"][mine].max()) + 1):
            sel = mine & (t["round"] == r)
            assert sel.any()
            want += 3 + int((t["sib_index"][sel] > 0).any())
    assert with_ghosts["n_buckets"] == want
    assert with_ghosts["n_rounds"] == t["round"].max() + 1
    assert without["n_buckets"] > want  # later siblings' ancestral cells sit at their parent's depth: extra batches


def test_capacity_parameters_and_repeated_runs():
    w = gen.drnn_workload(9, 32, 4, 32, seed=83)
    rc, t, st = A.acrobat_drnn_schedule(w)
    n = st["n_nodes"]
    assert rc == A.OK and n > 9
    for mode in MODES:
        assert A.acrobat_drnn_schedule(w, mode, True, max_nodes=n)[0] == A.OK
        rc, part, st2 = A.acrobat_drnn_schedule(w, mode, True, max_nodes=n - 1)
        assert rc == A.ENOMEM and st2["n_nodes"] == n - 1
    assert A.acrobat_drnn_schedule(dict(w, max_depth=0))[0] == A.EINVAL
    assert A.acrobat_drnn_schedule(dict(w, max_children=0))[0] == A.EINVAL
    assert A.acrobat_drnn_schedule(dict(w, max_depth=5000))[0] == A.EINVAL
    assert A.acrobat_drnn_schedule(dict(w, p_child=1.5))[0] == A.EINVAL
    assert A.acrobat_drnn_schedule(w, mode=7)[0] == A.EINVAL
    assert A.acrobat_drnn_schedule(dict(w, from_scores=True))[0] == A.EINVAL  # no scores without a GPU
    rc, t0, st0 = A.acrobat_drnn_schedule(dict(w, n_inst=0))
    assert rc == A.OK and st0["n_nodes"] == 0 and st0["n_rounds"] == 0
    # single nodes: roots that get no children
    rc, t1, st1 = A.acrobat_drnn_schedule(dict(w, max_depth=1))
    assert rc == A.OK and st1["n_nodes"] == 9 and st1["n_rounds"] == 1 and (t1["parent"] == -1).all()


def test_many_fibers_and_deep_recursion():
    """Thousands of fibers alive at once (every list of children is one), stacks reused by the next run."""
    w = gen.drnn_workload(300, 32, 7, 32, seed=84, max_depth=9, max_children=3, p_child=0.75, p_sibling=0.5, cap=200000)
    want = oracle.drnn(w)
    for _ in range(2):
        rc, got, st = A.acrobat_drnn_schedule(w, A.TDC_FORK_JOIN, True)
        assert rc == A.OK and st["n_nodes"] == len(want["inst"]) > 3000
        assert st["n_fibers"] > 800
    assert_same_trees(got, want)
    # depth-first generation of whole instances inside one fiber each: recursion max_depth deep
    rc, got, st = A.acrobat_drnn_schedule(w, A.TDC_INSTANCE_FIBERS, True)
    assert rc == A.OK
    assert_same_trees(got, want)


def fake_op(epi):
    p = 0x1000
    return B.acrobat_op_desc(epi, 64, 1, 64, p, 64, p, 64, p, 64, None, p, p, p, p, p, 0, p, 64, 1 << 30, 1 << 30, 1 << 30)


def test_ghost_operation_aligns_a_conditional():
    """Four instances; 0 and 1 run operator X then Y, 2 and 3 skip X (a conditional).  Eagerly, Y sits at depth 1
    for the first two and at depth 0 for the others: two batches.  A ghost on the short branch delays Y to
    depth 1 everywhere: one batch (the figure on ghost operators)."""
    for use_ghost, y_batches in ((False, 2), (True, 1)):
        g = A.Dfg(None)
        rc, X = g.acrobat_dfg_register_op_desc(fake_op(B.EPI_STORE_Z1))
        rc, Y = g.acrobat_dfg_register_op_desc(fake_op(B.EPI_RNN_STEP))
        y_nodes, ghosts = [], []
        for inst in range(4):
            if inst < 2:
                rc, x = g.acrobat_dfg_invoke(X, 0, 0, inst, inst)
                assert rc == A.OK
                rc, y = g.acrobat_dfg_invoke(Y, 0, 1, inst, inst, 0, x)
            elif use_ghost:
                rc, gh = g.acrobat_dfg_ghost(0, 0)
                assert rc == A.OK
                ghosts.append(gh)
                rc, y = g.acrobat_dfg_invoke(Y, 0, 1, inst, inst, 0, gh)
            else:
                rc, y = g.acrobat_dfg_invoke(Y, 0, 0, inst, inst)
            assert rc == A.OK
            y_nodes.append(y)
        off, order, bops = g.acrobat_dfg_schedule()
        assert int((bops == Y).sum()) == y_batches and int((bops == X).sum()) == 1
        assert sorted(order) == sorted(set(range(6 + len(ghosts))) - set(ghosts))  # ghosts are never scheduled
        assert set(y_nodes) <= set(order)
        g.close()


def test_ghost_depth_is_checked_like_any_node():
    g = A.Dfg(None)
    rc, X = g.acrobat_dfg_register_op_desc(fake_op(B.EPI_STORE_Z1))
    rc, x = g.acrobat_dfg_invoke(X, 0, 2, 0, 0)
    assert g.acrobat_dfg_ghost(0, 2, x)[0] == A.ESTRUCT  # not deeper than its producer
    rc, gh = g.acrobat_dfg_ghost(0, 3, x)
    assert rc == A.OK
    assert g.acrobat_dfg_invoke(X, 0, 3, 1, 1, 0, gh)[0] == A.ESTRUCT  # a consumer must come after the ghost
    assert g.acrobat_dfg_invoke(X, 0, 4, 1, 1, 0, gh)[0] == A.OK
    assert g.acrobat_dfg_ghost(0, 1, 99)[0] == A.ESTRUCT
    g.close()


@pytest.mark.parametrize("mode", MODES)
def test_a_chain_as_deep_as_allowed(mode):
    """One child per node down to the deepest level: the recursion nests 4096 calls on one stack."""
    w = gen.drnn_workload(2, 32, 3, 32, seed=85, max_depth=4096, max_children=1, p_child=1.0, p_sibling=1.0, cap=8192)
    rc, t, st = A.acrobat_drnn_schedule(w, mode, True)
    assert rc == A.OK and st["n_nodes"] == 8192 and t["depth"].max() == 4095
    assert st["n_rounds"] == (8192 if mode == A.TDC_SEQUENTIAL else 4096)
