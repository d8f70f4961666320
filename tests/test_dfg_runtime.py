"""Generic dataflow-graph runtime, host side (no GPU): buckets against the phase-schedule oracle,
the check of inline depths, the unbatched TreeLSTM program."""
import numpy as np
import pytest

import oracle
import paper_2305_10611_amd as A
from paper_2305_10611_amd import binding as B
from workloads import generators as gen


def fake_op(epi, nseg=1, H=64):
    """A descriptor with dummy non-null pointers: enough to build and schedule a graph."""
    p = 0x1000
    return B.acrobat_op_desc(epi, H, nseg, 64 if nseg else 0, p, 64, p, 64, p, 64 * max(nseg, 1), None, p, p, p, p, p,
                             H if epi == B.EPI_RELU_OUT else 0, p, H, 1 << 30, 1 << 30, 1 << 30)


def split_by_op(order, batch_off, ops_of_node):
    """Refines oracle batches (phase, depth) by op id, keeping ascending node ids."""
    off, out, bops = [0], [], []
    for b in range(len(batch_off) - 1):
        ids = order[batch_off[b]:batch_off[b + 1]]
        for op in sorted(set(ops_of_node[i] for i in ids)):
            sel = [i for i in ids if ops_of_node[i] == op]
            out += sel
            off.append(len(out))
            bops.append(op)
    return np.array(off), np.array(out), np.array(bops)


def test_treelstm_program_buckets_match_the_schedule_oracle():
    rng = gen.make_rng(5)
    trees = gen.tree_batch(rng.integers(1, 30, size=40), rng)
    trees, _ = gen.relabel_trees(trees, rng)
    trees["token"] = np.zeros(int(trees["tree_off"][-1]), np.int32)
    g = A.Dfg(None)
    rc, leaf = g.acrobat_dfg_register_op_desc(fake_op(B.EPI_TREE_LEAF))
    assert rc == A.OK
    rc, internal = g.acrobat_dfg_register_op_desc(fake_op(B.EPI_TREE_INTERNAL, nseg=2))
    assert rc == A.OK
    assert g.acrobat_dfg_build_treelstm(trees, 1, leaf, internal) == A.OK
    off, order, bops = g.acrobat_dfg_schedule()
    # node ids are in program order; compare through the arena rows (= global tree node ids)
    level_off, level_nodes, _, _ = oracle.tree_schedule(trees)
    assert np.array_equal(off, level_off)
    assert list(bops) == [leaf] + [internal] * (len(level_off) - 2)
    N = int(trees["tree_off"][-1])
    # program order = tree by tree, post-order: rebuild node id -> arena row the same way
    rows = []
    for t in range(trees["n_trees"]):
        b, e = int(trees["tree_off"][t]), int(trees["tree_off"][t + 1])
        child = set(trees["left"][b:e][trees["left"][b:e] >= 0]) | set(trees["right"][b:e][trees["right"][b:e] >= 0])
        root = [j for j in range(e - b) if j not in child][0]
        def post(j):
            if trees["left"][b + j] >= 0:
                post(int(trees["left"][b + j])); post(int(trees["right"][b + j]))
            rows.append(b + j)
        post(root)
    rows = np.array(rows)
    assert len(rows) == N
    for lv in range(len(level_off) - 1):
        got = sorted(rows[order[off[lv]:off[lv + 1]]])
        assert got == list(level_nodes[level_off[lv]:level_off[lv + 1]])
    g.close()


def test_birnn_graph_with_phases_matches_the_phase_schedule_oracle():
    from tests.test_oracle_birnn import birnn_graph
    lens = np.array([3, 1, 4, 0, 2, 6], np.int32)
    prods, R = birnn_graph(lens)
    phase = np.array([0] * (2 * R) + [1] * R, np.int32)
    depth, order_o, batch_off = oracle.phase_schedule(prods, phase)
    g = A.Dfg(None)
    ops = [g.acrobat_dfg_register_op_desc(fake_op(e))[1] for e in (B.EPI_RNN_STEP, B.EPI_RNN_STEP, B.EPI_RELU_OUT)]
    # the program inserts nodes in a valid program order (producers first); node id n of the oracle graph
    # gets inserted at position pos[n]
    ins = sorted(range(3 * R), key=lambda n: (phase[n], depth[n], n))
    pos = {n: i for i, n in enumerate(ins)}
    for n in ins:
        pr = [pos[p] for p in prods[n]] + [-1, -1]
        rc, node = g.acrobat_dfg_invoke(ops[n // R], int(phase[n]), int(depth[n]), n % R, 0, 0, pr[0], pr[1])
        assert rc == A.OK and node == pos[n]
    off, order, bops = g.acrobat_dfg_schedule()
    ops_of_node = {pos[n]: ops[n // R] for n in range(3 * R)}
    order_in_pos = np.array([pos[n] for n in order_o])
    # oracle batches hold ascending oracle ids; inside a (phase, depth, op) bucket the insertion order is the same
    e_off, e_order, e_ops = split_by_op(order_in_pos, batch_off, ops_of_node)
    assert np.array_equal(off, e_off) and np.array_equal(bops, e_ops)
    for b in range(len(off) - 1):
        assert sorted(order[off[b]:off[b + 1]]) == sorted(e_order[off[b]:off[b + 1]])
        assert list(order[off[b]:off[b + 1]]) == sorted(order[off[b]:off[b + 1]])
    # all output operators form ONE bucket although they hang behind recurrences of different lengths
    assert bops[-1] == ops[2] and off[-1] - off[-2] == R
    g.close()


def test_inline_depth_is_checked_against_the_producers():
    g = A.Dfg(None)
    _, op = g.acrobat_dfg_register_op_desc(fake_op(B.EPI_RNN_STEP))
    rc, a = g.acrobat_dfg_invoke(op, 0, 0, 0)
    assert rc == A.OK
    rc, b = g.acrobat_dfg_invoke(op, 0, 1, 1, 0, 0, a)
    assert rc == A.OK
    assert g.acrobat_dfg_invoke(op, 0, 1, 2, 1, 0, b)[0] == A.ESTRUCT        # same depth as its producer
    assert "does not come after" in g.acrobat_dfg_last_error()
    assert g.acrobat_dfg_invoke(op, 0, 0, 2, 1, 0, b)[0] == A.ESTRUCT        # shallower
    assert g.acrobat_dfg_invoke(op, 1, 0, 2, 1, 0, b)[0] == A.OK             # a later phase restarts at depth 0
    assert g.acrobat_dfg_invoke(op, 0, 5, 3, 0, 0, 2)[0] == A.ESTRUCT        # earlier phase than its producer
    assert g.acrobat_dfg_invoke(op, 0, 2, 3, 0, 0, 99)[0] == A.ESTRUCT       # producer does not exist yet
    assert g.acrobat_dfg_invoke(7, 0, 0, 0)[0] == A.EINVAL                   # unknown op
    assert g.acrobat_dfg_invoke(op, 0, 0, -1)[0] == A.EINVAL
    off, order, _ = g.acrobat_dfg_schedule()
    assert list(order) == [0, 1, 2] and list(off) == [0, 1, 2, 3]
    assert g.acrobat_dfg_run() == A.EINVAL                                   # no context
    g.acrobat_dfg_clear()
    assert list(g.acrobat_dfg_schedule()[0]) == [0]
    g.close()


def test_malformed_ops_and_trees_are_rejected():
    g = A.Dfg(None)
    bad = fake_op(B.EPI_TREE_LEAF)
    bad.H = 48
    assert g.acrobat_dfg_register_op_desc(bad)[0] == A.EINVAL
    bad = fake_op(B.EPI_TREE_INTERNAL, nseg=1)
    assert g.acrobat_dfg_register_op_desc(bad)[0] == A.EINVAL
    ok = fake_op(B.EPI_RNN_STEP)
    ok.zadd = None  # an RNN step without a hoisted input term
    assert g.acrobat_dfg_register_op_desc(ok)[0] == A.OK
    bad = fake_op(B.EPI_RNN_STEP)
    bad.h = None
    assert g.acrobat_dfg_register_op_desc(bad)[0] == A.EINVAL
    bad = fake_op(B.EPI_LSTM_STEP)
    bad.zadd = None
    assert g.acrobat_dfg_register_op_desc(bad)[0] == A.EINVAL
    _, leaf = g.acrobat_dfg_register_op_desc(fake_op(B.EPI_TREE_LEAF))
    _, internal = g.acrobat_dfg_register_op_desc(fake_op(B.EPI_TREE_INTERNAL, nseg=2))
    one_child = dict(n_trees=1, tree_off=np.array([0, 2], np.int32), left=np.array([-1, 0], np.int32),
                     right=np.array([-1, -1], np.int32), token=np.zeros(2, np.int32))
    assert g.acrobat_dfg_build_treelstm(one_child, 1, leaf, internal) == A.ESTRUCT
    two_roots = dict(n_trees=1, tree_off=np.array([0, 2], np.int32), left=np.array([-1, -1], np.int32),
                     right=np.array([-1, -1], np.int32), token=np.zeros(2, np.int32))
    assert g.acrobat_dfg_build_treelstm(two_roots, 1, leaf, internal) == A.ESTRUCT
    cyc = dict(n_trees=1, tree_off=np.array([0, 4], np.int32), left=np.array([-1, 2, 1, -1], np.int32),
               right=np.array([-1, 3, 0, -1], np.int32), token=np.zeros(4, np.int32))  # 1 <-> 2 cycle, no root... 
    assert g.acrobat_dfg_build_treelstm(cyc, 1, leaf, internal) == A.ESTRUCT
    tok = dict(n_trees=1, tree_off=np.array([0, 1], np.int32), left=np.array([-1], np.int32),
               right=np.array([-1], np.int32), token=np.array([5], np.int32))
    assert g.acrobat_dfg_build_treelstm(tok, 3, leaf, internal) == A.ESTRUCT
    g.close()


def test_matrix_vector_cell_op_takes_leaf_codes():
    g = A.Dfg(None)
    p = 0x1000
    mv = B.acrobat_op_desc(B.EPI_MVRNN, 64, 0, 0, p, 0, p, 0, p, 0, None, p, p, None, None, None, 0, None, 0, 10, 0, 25, p)
    rc, op = g.acrobat_dfg_register_op_desc(mv)
    assert rc == A.OK
    for field, value in (("H", 96), ("nseg", 1), ("W2", None), ("src1", None), ("c", None), ("src0_rows", 0)):
        bad = B.acrobat_op_desc.from_buffer_copy(mv)
        setattr(bad, field, value)
        assert g.acrobat_dfg_register_op_desc(bad)[0] == A.EINVAL, field
    # children: arena rows 0 .. 24 or leaf codes -1 .. -10 (table rows 0 .. 9)
    rc, n0 = g.acrobat_dfg_invoke(op, 0, 1, 0, -1, -10)
    assert rc == A.OK
    rc, n1 = g.acrobat_dfg_invoke(op, 0, 2, 1, 0, -3, n0)
    assert rc == A.OK
    assert g.acrobat_dfg_invoke(op, 0, 1, 2, -11, -1)[0] == A.EINVAL
    assert g.acrobat_dfg_invoke(op, 0, 1, 2, 25, -1)[0] == A.EINVAL
    assert g.acrobat_dfg_invoke(op, 0, 1, 25, -1, -1)[0] == A.EINVAL
    assert g.acrobat_dfg_invoke(op, 0, 2, 2, 0, 0, n1)[0] == A.ESTRUCT  # not deeper than its producer
    rc, other = g.acrobat_dfg_register_op_desc(fake_op(B.EPI_TREE_LEAF))
    assert g.acrobat_dfg_invoke(other, 0, 0, 0, -1)[0] == A.EINVAL  # other ops take no negative rows
    off, order, bops = g.acrobat_dfg_schedule()
    assert list(order) == [n0, n1] and list(bops) == [op, op]
    g.close()
