"""Pins for the bidirectional-RNN oracle and the phase-aware schedule oracle."""
import numpy as np
import pytest
import torch

import oracle
from workloads import generators as gen


def test_two_step_hand_value(golden):
    g = golden("hand_cases.txt")
    w = dict(n_seq=1, len=np.array([2], np.int32), H=1, D=1, n_out=2, x=np.array([[1.0], [-1.0]], np.float32),
             fWx=[[1.0]], fWh=[[0.5]], fb=[0.0], finit=[0.25], bWx=[[-1.0]], bWh=[[2.0]], bb=[0.5], binit=[0.75],
             C=[[2.0, -0.5], [1.0, -2.0]], cb=[0.25, 0.25])
    hf, hb, y = oracle.birnn(w)
    np.testing.assert_allclose(hf[:, 0], g["birnn_hf"], atol=1e-15)
    np.testing.assert_allclose(hb[:, 0], g["birnn_hb"], atol=1e-15)
    np.testing.assert_allclose(y[0], g["birnn_y0"], atol=1e-15)
    np.testing.assert_allclose(y[1], g["birnn_y1"], atol=1e-15)


def test_matches_library_bidirectional_rnn():
    """s(z) = (1 + tanh(z/2)) / 2, so with g = 2h - 1 the sigmoid cell is the library's tanh RNN with
    W_ih = Wx/2, W_hh = Wh/4, bias = b/2 + (Wh 1)/4, g_init = 2 h_init - 1; the library's bidirectional
    mode also supplies the reversed pass and the [forward ; backward] concatenation."""
    w = gen.birnn_workload(7, 0, 11, 12, 9, 5, seed=61, bias_scale=0.4)
    H, D = w["H"], w["D"]
    hf, hb, y = oracle.birnn(w)
    rnn = torch.nn.RNN(D, H, nonlinearity="tanh", bias=True, batch_first=True, bidirectional=True, dtype=torch.float64)
    f64 = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    with torch.no_grad():
        for sfx, p in (("", "f"), ("_reverse", "b")):
            Wh = w[p + "Wh"].astype(np.float64)
            getattr(rnn, "weight_ih_l0" + sfx).copy_(f64(w[p + "Wx"]) / 2)
            getattr(rnn, "weight_hh_l0" + sfx).copy_(f64(Wh) / 4)
            getattr(rnn, "bias_ih_l0" + sfx).copy_(f64(w[p + "b"]) / 2 + f64(Wh.sum(axis=1)) / 4)
            getattr(rnn, "bias_hh_l0" + sfx).zero_()
        g0 = torch.stack([2 * f64(w["finit"]) - 1, 2 * f64(w["binit"]) - 1])[:, None, :]  # [2, 1, H]
        for s in range(w["n_seq"]):
            b, e = int(w["seq_off"][s]), int(w["seq_off"][s + 1])
            if e == b:
                continue
            out, _ = rnn(f64(w["x"][b:e])[None], g0)
            hcat = (out[0] + 1) / 2  # [T, 2H]
            np.testing.assert_allclose(hf[b:e], hcat[:, :H].numpy(), rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(hb[b:e], hcat[:, H:].numpy(), rtol=1e-12, atol=1e-13)
            want_y = torch.relu(torch.nn.functional.linear(hcat, f64(w["C"]), f64(w["cb"])))
            np.testing.assert_allclose(y[b:e], want_y.numpy(), rtol=1e-12, atol=1e-13)


def test_reversing_the_input_swaps_the_directions():
    w = gen.birnn_workload(4, 1, 9, 6, 5, 3, seed=62)
    hf, hb, y = oracle.birnn(w)
    w2 = dict(w)
    x2 = w["x"].copy()
    for s in range(w["n_seq"]):
        b, e = int(w["seq_off"][s]), int(w["seq_off"][s + 1])
        x2[b:e] = w["x"][b:e][::-1]
    w2["x"] = x2
    for k in ("Wx", "Wh", "b", "init"):
        w2["f" + k], w2["b" + k] = w["b" + k], w["f" + k]
    H = w["H"]
    w2["C"] = np.concatenate([w["C"][:, H:], w["C"][:, :H]], axis=1)
    hf2, hb2, y2 = oracle.birnn(w2)
    for s in range(w["n_seq"]):
        b, e = int(w["seq_off"][s]), int(w["seq_off"][s + 1])
        assert np.array_equal(hf2[b:e], hb[b:e][::-1]) and np.array_equal(hb2[b:e], hf[b:e][::-1])
        np.testing.assert_allclose(y2[b:e], y[b:e][::-1], rtol=1e-13, atol=1e-15)


def test_independence_threads_and_zero_weights():
    w = gen.birnn_workload(6, 0, 8, 5, 4, 3, seed=63)
    hf, hb, y = oracle.birnn(w)
    hf2, hb2, y2 = oracle.birnn(w, nthreads=3)
    assert np.array_equal(hf, hf2) and np.array_equal(hb, hb2) and np.array_equal(y, y2)
    s = int(np.argmax(w["len"]))
    b, e = int(w["seq_off"][s]), int(w["seq_off"][s + 1])
    w1 = dict(w, n_seq=1, len=w["len"][s:s + 1], x=w["x"][b:e])
    hf1, hb1, y1 = oracle.birnn(w1)
    assert np.array_equal(hf1, hf[b:e]) and np.array_equal(hb1, hb[b:e]) and np.array_equal(y1, y[b:e])
    for k in ("fWx", "fWh", "bWx", "bWh"):
        w[k] = np.zeros_like(w[k])
    hf, hb, y = oracle.birnn(w)
    sg = lambda t: 1.0 / (1.0 + np.exp(-t))
    np.testing.assert_allclose(hf, np.broadcast_to(sg(w["fb"].astype(np.float64)), hf.shape), rtol=1e-15)
    np.testing.assert_allclose(hb, np.broadcast_to(sg(w["bb"].astype(np.float64)), hb.shape), rtol=1e-15)


# ---------------------------------------------------------------- phase-aware schedule
def birnn_graph(lens):
    """Explicit dataflow graph of the BiRNN: node ids  fwd(s,t) = row, bwd(s,t) = R + row,
    out(s,t) = 2R + row;  the recurrences are phase 0, the output operators phase 1."""
    off = np.concatenate([[0], np.cumsum(lens)])
    R = int(off[-1])
    prods = [[] for _ in range(3 * R)]
    for s, T in enumerate(lens):
        for t in range(T):
            r = int(off[s]) + t
            if t > 0:
                prods[r].append(r - 1)
            if t < T - 1:
                prods[R + r].append(R + r + 1)
            prods[2 * R + r] += [r, R + r]
    return prods, R


def test_phase_schedule_of_the_birnn_graph():
    lens = np.array([3, 1, 4, 0, 2], np.int32)
    prods, R = birnn_graph(lens)
    phase = np.array([0] * (2 * R) + [1] * R, np.int32)
    depth, order, batch_off = oracle.phase_schedule(prods, phase)
    off = np.concatenate([[0], np.cumsum(lens)])
    # recurrences: depth = steps already taken in their direction; outputs: all depth 0 of phase 1
    for s, T in enumerate(lens):
        for t in range(T):
            r = off[s] + t
            assert depth[r] == t and depth[R + r] == T - 1 - t and depth[2 * R + r] == 0
    assert len(batch_off) - 1 == lens.max() + 1  # one batch per step, then ONE batch of all outputs
    assert list(order[batch_off[-2]:]) == list(range(2 * R, 3 * R))
    # without phases the output operators are spread over many depths (the eagerness the paper fixes)
    depth1, _, batch_off1 = oracle.phase_schedule(prods, np.zeros(3 * R, np.int32))
    assert len(set(depth1[2 * R:])) > 1
    # brute force: depth by longest same-phase producer chain
    def brute(n):
        same = [p for p in prods[n] if phase[p] == phase[n]]
        return 0 if not same else 1 + max(brute(p) for p in same)
    assert [brute(n) for n in range(3 * R)] == list(depth)


def test_phase_schedule_reduces_to_tree_depths_with_one_phase():
    rng = gen.make_rng(64)
    trees = gen.tree_batch(rng.integers(1, 12, size=9), rng)
    trees, _ = gen.relabel_trees(trees, rng)
    base = np.repeat(trees["tree_off"][:-1], np.diff(trees["tree_off"]))
    prods = [[] if l < 0 else [int(b + l), int(b + r)] for l, r, b in zip(trees["left"], trees["right"], base)]
    depth, order, batch_off = oracle.phase_schedule(prods, np.zeros(len(prods), np.int32))
    n_levels, tdepth = oracle.tree_depths(trees)
    assert np.array_equal(depth, tdepth)
    level_off, level_nodes, _, _ = oracle.tree_schedule(trees)
    assert np.array_equal(order, level_nodes) and np.array_equal(batch_off, level_off)
