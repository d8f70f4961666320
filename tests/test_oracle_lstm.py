"""Pins for the variable-length LSTM oracle: hand values, library LSTM, padding invariance."""
import numpy as np
import pytest
import torch

import oracle
from workloads import generators as gen


def test_two_step_hand_value(golden):
    g = golden("hand_cases.txt")
    w = dict(n_seq=1, len=np.array([2], np.int32), H=1, D=1, x=np.array([[1.0], [-1.0]], np.float32),
             Wx=np.ones((4, 1), np.float32), Wh=np.full((4, 1), 0.5, np.float32), b=np.zeros(4, np.float32))
    h, c = oracle.varlen_lstm(w)
    assert c[0, 0] == pytest.approx(g["lstm_c0"], abs=1e-15)
    assert h[0, 0] == pytest.approx(g["lstm_h0"], abs=1e-15)
    assert c[1, 0] == pytest.approx(g["lstm_c1"], abs=1e-15)
    assert h[1, 0] == pytest.approx(g["lstm_h1"], abs=1e-14)


def test_matches_library_lstm_sequence_by_sequence():
    w = gen.lstm_workload(6, 0, 9, 12, 10, seed=21, bias_scale=0.4)
    H, D = w["H"], w["D"]
    h, c = oracle.varlen_lstm(w)
    rows = lambda M, g: M[g * H:(g + 1) * H]
    # library order (i, f, g, o); ours (i, f, o, u)
    pick = lambda M: np.concatenate([rows(M, 0), rows(M, 1), rows(M, 3), rows(M, 2)]).astype(np.float64)
    lstm = torch.nn.LSTM(D, H, num_layers=1, bias=True, batch_first=True, dtype=torch.float64)
    with torch.no_grad():
        lstm.weight_ih_l0.copy_(torch.from_numpy(pick(w["Wx"])))
        lstm.weight_hh_l0.copy_(torch.from_numpy(pick(w["Wh"])))
        lstm.bias_ih_l0.copy_(torch.from_numpy(pick(w["b"])))
        lstm.bias_hh_l0.zero_()
        for s in range(w["n_seq"]):
            b, e = int(w["seq_off"][s]), int(w["seq_off"][s + 1])
            if e == b:
                continue
            x = torch.from_numpy(w["x"][b:e].astype(np.float64))[None]
            out, (hn, cn) = lstm(x)
            np.testing.assert_allclose(h[b:e], out[0].numpy(), rtol=1e-12, atol=1e-14)
            np.testing.assert_allclose(c[e - 1], cn[0, 0].numpy(), rtol=1e-12, atol=1e-14)


def test_a_sequence_does_not_depend_on_the_others():
    w = gen.lstm_workload(5, 1, 8, 6, 5, seed=22)
    h, c = oracle.varlen_lstm(w)
    h2, c2 = oracle.varlen_lstm(w, nthreads=3)
    assert np.array_equal(h, h2) and np.array_equal(c, c2)
    s = 3
    b, e = int(w["seq_off"][s]), int(w["seq_off"][s + 1])
    w1 = dict(w)
    w1.update(n_seq=1, len=w["len"][s:s + 1], x=w["x"][b:e])
    h1, c1 = oracle.varlen_lstm(w1)
    assert np.array_equal(h1, h[b:e]) and np.array_equal(c1, c[b:e])


def test_zero_weights():
    w = gen.lstm_workload(3, 1, 5, 4, 4, seed=23)
    w["Wx"] = np.zeros_like(w["Wx"])
    w["Wh"] = np.zeros_like(w["Wh"])
    h, c = oracle.varlen_lstm(w)
    assert np.all(h == 0) and np.all(c == 0)
