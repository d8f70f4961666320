"""Pins for the doubly-recurrent-network oracle (top-down tree generation with emulated
tensor-dependent decisions)."""
import numpy as np
import pytest
import torch

import oracle
from workloads import generators as gen

GOLDEN_RATIO_64 = 0x9E3779B97F4A7C15
M64 = 2**64 - 1


def test_generator_matches_published_splitmix64_outputs():
    # first three outputs of splitmix64 seeded with 0, as listed with its reference implementation
    want = (0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F)
    got = tuple(oracle.mix64((i * GOLDEN_RATIO_64) & M64) for i in range(3))
    assert got == want


def tiny(max_depth, max_children, **kw):
    w = dict(n_inst=1, H=1, n_labels=1, n_out=2, x0=[[0.5]], emb=[[2.0]], Wa=[[1.0, 0.5]], ba=[0.0], Wf=[[-1.0, 0.25]],
             bf=[0.125], Wp=[[2.0, -2.0]], bp=[0.0], Wo=[[1.0], [-1.0]], bo=[0.0, 0.5], seed_decisions=1, max_depth=max_depth,
             max_children=max_children, p_child=1.0, p_sibling=1.0, cap=64)
    w.update(kw)
    return w


def test_hand_values_root_with_two_children(golden):
    g = golden("hand_cases.txt")
    r = oracle.drnn(tiny(2, 2))
    assert r["parent"].tolist() == [-1, 0, 0] and r["prev"].tolist() == [-1, -1, 1]
    assert r["sib_index"].tolist() == [0, 0, 1] and r["depth"].tolist() == [0, 1, 1]
    tight = dict(rtol=0, atol=2e-16)
    np.testing.assert_allclose(r["a"][:, 0], g["drnn_a"], **tight)
    np.testing.assert_allclose(r["f"][:, 0], g["drnn_f"], **tight)
    np.testing.assert_allclose(r["g"][:, 0], g["drnn_g"], **tight)
    np.testing.assert_allclose(r["y"][:, 0], g["drnn_g"], **tight)
    np.testing.assert_allclose(r["y"][:, 1], 0.5 - np.asarray(g["drnn_g"]), **tight)


def library_sigmoid_rnn(Wx, Wh, b, init, x):
    """h_t = s(Wx x_t + b + Wh h_{t-1}) through the library's tanh RNN: s(z) = (1 + tanh(z/2)) / 2."""
    H, D = Wx.shape
    rnn = torch.nn.RNN(D, H, nonlinearity="tanh", bias=True, batch_first=True, dtype=torch.float64)
    f64 = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    with torch.no_grad():
        rnn.weight_ih_l0.copy_(f64(Wx) / 2)
        rnn.weight_hh_l0.copy_(f64(Wh) / 4)
        rnn.bias_ih_l0.copy_(f64(b) / 2 + f64(np.asarray(Wh, np.float64).sum(axis=1)) / 4)
        rnn.bias_hh_l0.zero_()
        out, _ = rnn(f64(x)[None], (2 * f64(init) - 1)[None, None])
    return ((out[0] + 1) / 2).numpy()


def test_single_child_chain_is_the_library_rnn_along_the_depth():
    """One child per node and one label: the ancestral states form a plain recurrent chain whose
    input is the label embedding at every step and whose initial state is the instance's vector."""
    H, L = 12, 9
    w = gen.drnn_workload(3, H, 1, 5, seed=71, max_depth=L, max_children=1, p_child=1.0, p_sibling=1.0, bias_scale=0.4)
    r = oracle.drnn(w)
    assert len(r["inst"]) == 3 * L
    x = np.repeat(w["emb"][:1], L, axis=0)
    for s in range(3):
        rows = np.nonzero(r["inst"] == s)[0]
        assert r["depth"][rows].tolist() == list(range(L))
        want = library_sigmoid_rnn(w["Wa"][:, H:], w["Wa"][:, :H], w["ba"], w["x0"][s], x)
        np.testing.assert_allclose(r["a"][rows], want, atol=1e-13)
        # every node is a first child: the fraternal state is the same constant everywhere
        f0 = library_sigmoid_rnn(w["Wf"][:, H:], w["Wf"][:, :H], w["bf"], np.zeros(H), x[:1])
        np.testing.assert_allclose(r["f"][rows], np.repeat(f0, L, axis=0), atol=1e-13)


def test_sibling_chain_is_the_library_rnn_along_the_siblings():
    """Two levels, every sibling slot used, one label: the children's fraternal states form a
    recurrent chain from a zero state (library initial state g = 2*0 - 1)."""
    H, C = 10, 7
    w = gen.drnn_workload(2, H, 1, 4, seed=72, max_depth=2, max_children=C, p_child=1.0, p_sibling=1.0, bias_scale=0.4)
    r = oracle.drnn(w)
    assert len(r["inst"]) == 2 * (C + 1)
    x = np.repeat(w["emb"][:1], C, axis=0)
    want = library_sigmoid_rnn(w["Wf"][:, H:], w["Wf"][:, :H], w["bf"], np.zeros(H), x)
    for s in range(2):
        rows = np.nonzero((r["inst"] == s) & (r["depth"] == 1))[0]
        assert r["sib_index"][rows].tolist() == list(range(C))
        np.testing.assert_allclose(r["f"][rows], want, atol=1e-13)


def test_predictive_state_and_scores_from_the_two_states():
    w = gen.drnn_workload(5, 16, 7, 6, seed=73, bias_scale=0.3)
    r = oracle.drnn(w)
    af = np.concatenate([r["a"], r["f"]], axis=1)
    g = 1.0 / (1.0 + np.exp(-(af @ w["Wp"].astype(np.float64).T + w["bp"])))
    np.testing.assert_allclose(r["g"], g, atol=1e-13)
    np.testing.assert_allclose(r["y"], g @ w["Wo"].astype(np.float64).T + w["bo"], atol=1e-13)
    # labels select the embedding row: a child's ancestral state changes if its parent's row is changed
    child = int(np.nonzero(r["parent"] >= 0)[0][0])
    w2 = dict(w)
    w2["emb"] = w["emb"].copy()
    w2["emb"][r["label"][r["parent"][child]]] += 1.0
    r2 = oracle.drnn(w2)
    assert np.abs(r2["a"][child] - r["a"][child]).max() > 1e-3


def paths(r):
    """(instance, child indices from the root) of every node."""
    out = []
    for i in range(len(r["inst"])):
        p, j = [], i
        while r["parent"][j] >= 0:
            p.append(int(r["sib_index"][j]))
            j = int(r["parent"][j])
        out.append((int(r["inst"][i]), tuple(reversed(p))))
    return out


def test_structure_follows_the_decisions_and_the_limits():
    w = gen.drnn_workload(40, 4, 9, 3, seed=74, max_depth=5, max_children=3, p_child=0.8, p_sibling=0.6)
    r = oracle.drnn(w)
    n = len(r["inst"])
    pth = paths(r)
    assert len(set(pth)) == n
    index = {p: i for i, p in enumerate(pth)}
    n_child = np.zeros(n, int)
    for i in range(n):
        inst, p = pth[i]
        assert r["depth"][i] == len(p) < w["max_depth"]
        assert r["sib_index"][i] == (p[-1] if p else 0) < w["max_children"]
        if p:
            assert r["parent"][i] == index[(inst, p[:-1])] < i  # pre-order: parents first
            assert r["prev"][i] == (index[(inst, p[:-1] + (p[-1] - 1,))] if p[-1] else -1)
            n_child[r["parent"][i]] += 1
        else:
            assert r["parent"][i] == -1 and r["prev"][i] == -1
    assert sorted(set(r["inst"].tolist())) == list(range(40))  # every instance has a root
    assert (np.diff(r["inst"]) >= 0).all()
    # every position has a key of its own (siblings, cousins, other instances): no two nodes share their decisions
    keys = [oracle.drnn_keys(w["seed_decisions"], inst, p) for inst, p in pth]
    assert len(set(keys)) == n
    assert oracle.drnn_keys(w["seed_decisions"] + 1, 0) != oracle.drnn_keys(w["seed_decisions"], 0)
    for i in range(n):
        inst, p = pth[i]
        has_child, has_sib, label = oracle.drnn_decide(oracle.drnn_keys(w["seed_decisions"], inst, p), len(p),
                                                       p[-1] if p else 0, not p, w)
        assert label == r["label"][i] and 0 <= label < w["n_labels"]
        assert has_child == (n_child[i] > 0)
        assert has_sib == ((inst, p[:-1] + (p[-1] + 1,)) in index if p else False)


def test_decision_rates_and_limits():
    w = dict(max_depth=4, max_children=3, p_child=0.3, p_sibling=0.75, n_labels=5)
    keys = [oracle.mix64(1000 + i) for i in range(20000)]
    d = np.array([oracle.drnn_decide(k, 1, 0, False, w) for k in keys])
    for col, p in ((0, 0.3), (1, 0.75)):
        assert abs(d[:, col].mean() - p) < 4 * np.sqrt(p * (1 - p) / len(keys))
    assert abs(np.corrcoef(d[:, 0], d[:, 1])[0, 1]) < 0.03
    cnt = np.bincount(d[:, 2], minlength=5)
    assert cnt.min() > 0.9 * len(keys) / 5 and len(cnt) == 5
    # the limits: no children on the last level, no sibling after the last slot, none for a root
    assert not any(oracle.drnn_decide(k, 3, 0, False, w)[0] for k in keys[:500])
    assert not any(oracle.drnn_decide(k, 1, 2, False, w)[1] for k in keys[:500])
    assert not any(oracle.drnn_decide(k, 0, 0, True, w)[1] for k in keys[:500])
    w1 = dict(w, p_child=1.0, p_sibling=1.0)
    assert all(oracle.drnn_decide(k, 2, 1, False, w1)[:2] == (1, 1) for k in keys[:500])


def test_instances_are_independent_and_capacity_is_checked():
    w = gen.drnn_workload(6, 8, 5, 4, seed=75)
    r = oracle.drnn(w)
    w3 = dict(w, n_inst=3, x0=w["x0"][:3])
    r3 = oracle.drnn(w3)
    n3 = len(r3["inst"])
    assert n3 == int((r["inst"] < 3).sum())
    for k in r3:
        np.testing.assert_array_equal(r3[k], r[k][:n3])
    with pytest.raises(ValueError):
        oracle.drnn(w, cap=len(r["inst"]) - 1)
    assert len(oracle.drnn(w, cap=len(r["inst"]))["inst"]) == len(r["inst"])


def test_hand_values_with_decisions_read_off_the_scores(golden):
    g = golden("hand_cases.txt")
    w = tiny(2, 3, n_labels=2, n_out=4, emb=[[2.0], [-1.0]], Wo=[[1.0], [1.0], [1.0], [-1.0]], bo=[0.0, -0.4375, 0.0, 1.25],
             from_scores=True, p_child=0.0, p_sibling=0.0)
    r = oracle.drnn(w)
    assert r["parent"].tolist() == [-1, 0, 0, 0] and r["prev"].tolist() == [-1, -1, 1, 2]
    assert r["label"].tolist() == [int(v) for v in g["drnn_scores_label"]]
    tight = dict(rtol=0, atol=2e-16)
    for k in "afg":
        np.testing.assert_allclose(r[k][:, 0], g["drnn_scores_" + k], **tight)
    # one level only: the root's y0 > 0 no longer gives it children
    assert len(oracle.drnn(dict(w, max_depth=1))["inst"]) == 1
    # a higher threshold on the sibling score: child 0 (g - 0.4688 < 0) stays alone
    assert oracle.drnn(dict(w, bo=[0.0, -0.46875, 0.0, 1.25]))["parent"].tolist() == [-1, 0]


def score_decisions(y, depth, k, is_root, w):
    n = min(int(w["n_labels"]), int(w["n_out"]) - 2)
    return (depth + 1 < w["max_depth"] and y[0] > 0, (not is_root) and k + 1 < w["max_children"] and y[1] > 0,
            int(np.argmax(y[2:2 + n])))


def test_score_driven_structure_follows_the_scores():
    w = gen.drnn_workload(24, 64, 30, 32, seed=128, from_scores=True)
    r = oracle.drnn(w)
    n = len(r["inst"])
    sizes = np.bincount(r["inst"], minlength=24)
    # this seed grows trees of several sizes with several labels (checked, not assumed)
    assert n > 300 and len(set(sizes.tolist())) >= 4 and sizes.max() > 20 and len(set(r["label"].tolist())) >= 3
    pth = paths(r)
    index = {p: i for i, p in enumerate(pth)}
    n_child = np.bincount(r["parent"][r["parent"] >= 0], minlength=n)
    for i, (inst, p) in enumerate(pth):
        has_child, has_sib, label = score_decisions(r["y"][i], len(p), p[-1] if p else 0, not p, w)
        assert label == r["label"][i]
        assert has_child == (n_child[i] > 0)
        assert has_sib == ((inst, p[:-1] + (p[-1] + 1,)) in index if p else False)


def test_scores_that_always_say_yes_grow_the_full_tree_of_the_emulation():
    """Topology scores forced positive = emulated decisions with probability one (one label, so labels agree)."""
    w = gen.drnn_workload(3, 8, 1, 3, seed=76, max_depth=4, max_children=3, p_child=1.0, p_sibling=1.0)
    full = oracle.drnn(w)
    assert len(full["inst"]) == 3 * (1 + 3 + 9 + 27)
    ws = dict(w, from_scores=True, Wo=w["Wo"].copy(), bo=w["bo"].copy())
    ws["Wo"][:2] = 0.0
    ws["bo"][:2] = 1.0
    got = oracle.drnn(ws)
    for k in ("inst", "parent", "prev", "sib_index", "depth", "label"):
        assert np.array_equal(got[k], full[k])
    for k in "afg":
        assert np.array_equal(got[k], full[k])
    ws["bo"][0] = -1.0  # ... and with the first score forced negative nobody has children
    assert len(oracle.drnn(ws)["inst"]) == 3
