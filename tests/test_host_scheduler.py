"""Host logic of the product library (no GPU): exported symbols, level scheduler vs the
schedule oracle (bit exact), rejection of malformed structures."""
import os
import re

import numpy as np
import pytest

import oracle
import paper_2305_10611_amd as A
from workloads import generators as gen
from workloads import make_config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "acrobat.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(acrobat_[a-z_]+)\s*\(", text))
    assert declared == set(A.EXPORTS)
    for name in declared:
        assert hasattr(A.lib, name), name


def test_library_exports_nothing_but_the_declared_c_abi():
    """Hidden visibility + the linker's version script: no C++ internals leak out of the shared library."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", A.binding._build.LIB], capture_output=True, text=True, check=True).stdout
    names = {line.split()[-1] for line in out.splitlines() if line.strip()}
    assert names == set(A.EXPORTS), sorted(names ^ set(A.EXPORTS))


@pytest.mark.parametrize("cfg", [0, 1, 2, 3])
def test_tree_schedule_is_bit_exact_on_benchmark_configs(cfg):
    w = make_config(cfg)
    rc, level_off, level_nodes, lrow, rrow = A.acrobat_schedule_trees(w, w["V"])
    assert rc == A.OK
    o_off, o_nodes, o_l, o_r = oracle.tree_schedule(w)
    assert np.array_equal(level_off, o_off) and np.array_equal(level_nodes, o_nodes)
    assert np.array_equal(lrow, o_l) and np.array_equal(rrow, o_r)


@pytest.mark.parametrize("seed", range(5))
def test_tree_schedule_is_bit_exact_under_random_numbering(seed):
    rng = gen.make_rng(1000 + seed)
    trees = gen.tree_batch(rng.integers(1, 40, size=30), rng)
    trees, _ = gen.relabel_trees(trees, rng)
    rc, level_off, level_nodes, lrow, rrow = A.acrobat_schedule_trees(trees)
    assert rc == A.OK
    o_off, o_nodes, o_l, o_r = oracle.tree_schedule(trees)
    assert np.array_equal(level_off, o_off) and np.array_equal(level_nodes, o_nodes)
    assert np.array_equal(lrow, o_l) and np.array_equal(rrow, o_r)


def test_deep_chain_and_empty_inputs():
    # a 3000-leaf left chain: 3000 levels, no recursion limit in the product scheduler
    L = 3000
    n = 2 * L - 1
    left = np.full(n, -1, np.int32)
    right = np.full(n, -1, np.int32)
    for t in range(L - 1):
        left[L + t] = 0 if t == 0 else L + t - 1
        right[L + t] = t + 1
    trees = dict(n_trees=1, tree_off=np.array([0, n], np.int32), left=left, right=right)
    rc, level_off, level_nodes, _, _ = A.acrobat_schedule_trees(trees)
    assert rc == A.OK and len(level_off) - 1 == L and level_off[1] == L
    assert list(level_nodes[L:]) == list(range(L, n))
    # empty batch, and a batch containing empty trees
    rc, level_off, level_nodes, _, _ = A.acrobat_schedule_trees(
        dict(n_trees=0, tree_off=np.array([0], np.int32), left=np.zeros(0, np.int32), right=np.zeros(0, np.int32)))
    assert rc == A.OK and list(level_off) == [0]
    rc, level_off, level_nodes, _, _ = A.acrobat_schedule_trees(
        dict(n_trees=3, tree_off=np.array([0, 0, 1, 1], np.int32), left=np.array([-1], np.int32),
             right=np.array([-1], np.int32)))
    assert rc == A.OK and list(level_off) == [0, 1] and list(level_nodes) == [0]


def _one(left, right, token=None, vocab=-1, tree_off=None):
    left = np.asarray(left, np.int32)
    t = dict(n_trees=1 if tree_off is None else len(tree_off) - 1,
             tree_off=np.asarray([0, len(left)] if tree_off is None else tree_off, np.int32), left=left,
             right=np.asarray(right, np.int32), token=None if token is None else np.asarray(token, np.int32))
    return A.acrobat_schedule_trees(t, vocab)[0]


def test_malformed_structures_are_rejected():
    assert _one([-1, -1, 0], [-1, -1, 1]) == A.OK
    assert _one([-1, -1, 0], [-1, -1, -1]) == A.ESTRUCT   # exactly one child
    assert _one([-1, -1, 0], [-1, -1, 3]) == A.ESTRUCT    # child out of range
    assert _one([-1, -1, -2], [-1, -1, 1]) == A.ESTRUCT   # negative other than -1
    assert _one([-1, -1, 0], [-1, -1, 0]) == A.ESTRUCT    # same child twice
    assert _one([-1, -1, 2], [-1, -1, 1]) == A.ESTRUCT    # own child
    assert _one([-1, -1, 0, 0], [-1, -1, 1, 1]) == A.ESTRUCT  # two parents
    assert _one([-1, -1, -1], [-1, -1, -1]) == A.ESTRUCT  # three roots
    # a 2-cycle next to a proper root: 0 leaf,1 leaf; 2=(0,3) 3=(2,1)?? -> 2 and 3 are each other's child
    assert _one([-1, -1, 0, 2], [-1, -1, 3, 1]) == A.ESTRUCT
    # cycle hanging beside a valid tree: nodes 0,1,2 valid; 3=(4,5) 4=(3,6) 5,6 leaves -> no second root
    assert _one([-1, -1, 0, 4, 3, -1, -1], [-1, -1, 1, 5, 6, -1, -1]) == A.ESTRUCT
    # tokens
    assert _one([-1, -1, 0], [-1, -1, 1], token=[0, 4, -1], vocab=5) == A.OK
    assert _one([-1, -1, 0], [-1, -1, 1], token=[0, 5, -1], vocab=5) == A.ESTRUCT
    assert _one([-1, -1, 0], [-1, -1, 1], token=[-1, 2, 0], vocab=5) == A.ESTRUCT
    # child index must be local to its own tree
    assert _one([-1, -1, 0, -1], [-1, -1, 3, -1], tree_off=[0, 3, 4]) == A.ESTRUCT
    # tree_off not starting at 0 / decreasing
    assert _one([-1], [-1], tree_off=[1, 1]) == A.EINVAL
    assert _one([-1, -1], [-1, -1], tree_off=[0, 2, 1]) == A.EINVAL


@pytest.mark.parametrize("seed", range(3))
def test_sequence_schedule_is_bit_exact(seed):
    rng = gen.make_rng(2000 + seed)
    lens = rng.integers(0, 50, size=37).astype(np.int32)
    rc, level_off, rows = A.acrobat_schedule_seqs(lens)
    assert rc == A.OK
    o_off, o_rows = oracle.seq_schedule(lens)
    assert np.array_equal(level_off, o_off) and np.array_equal(rows, o_rows)


def test_sequence_schedule_edge_cases():
    rc, level_off, rows = A.acrobat_schedule_seqs(np.zeros(0, np.int32))
    assert rc == A.OK and list(level_off) == [0]
    rc, level_off, rows = A.acrobat_schedule_seqs(np.zeros(4, np.int32))
    assert rc == A.OK and list(level_off) == [0] and rows.size == 0
    assert A.acrobat_schedule_seqs(np.array([3, -1], np.int32))[0] == A.EINVAL
    w = make_config(4)
    rc, level_off, rows = A.acrobat_schedule_seqs(w["len"])
    sizes = np.diff(level_off)
    assert sizes[0] == (w["len"] > 0).sum() and sizes.sum() == w["len"].sum() and np.all(np.diff(sizes) <= 0)


# ---------------------------------------------------------------- bidirectional RNN with phases
@pytest.mark.parametrize("lens", [[3, 1, 4, 0, 2], [1], [0, 0], [], [7, 7, 7], [1, 9, 2, 9, 1, 0, 5]])
def test_birnn_schedule_is_bit_exact_against_the_phase_schedule_oracle(lens):
    from tests.test_oracle_birnn import birnn_graph
    lens = np.asarray(lens, np.int32)
    rc, level_off, level_codes = A.acrobat_schedule_birnn(lens)
    assert rc == A.OK
    prods, R = birnn_graph(lens)
    if R == 0:
        assert list(level_off) == [0] and level_codes.size == 0
        return
    phase = np.array([0] * (2 * R) + [1] * R, np.int32)
    _, order, batch_off = oracle.phase_schedule(prods, phase)
    assert np.array_equal(level_off, batch_off) and np.array_equal(level_codes, order)


def test_birnn_schedule_on_a_random_batch_and_bad_input():
    rng = gen.make_rng(77)
    lens = rng.integers(0, 40, size=200).astype(np.int32)
    from tests.test_oracle_birnn import birnn_graph
    rc, level_off, level_codes = A.acrobat_schedule_birnn(lens)
    assert rc == A.OK
    prods, R = birnn_graph(lens)
    _, order, batch_off = oracle.phase_schedule(prods, np.array([0] * (2 * R) + [1] * R, np.int32))
    assert np.array_equal(level_off, batch_off) and np.array_equal(level_codes, order)
    rc, _, _ = A.acrobat_schedule_birnn(np.array([3, -1], np.int32))
    assert rc == A.ESTRUCT or rc == A.EINVAL
