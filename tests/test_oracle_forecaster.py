"""Pins for the CPU oracle of the service workload predictor's online phase (paper Sec. 3.2, Alg. 2)."""
import os

import numpy as np
import torch

from oracle import forecaster as of


def random_model(rng, hm):
    w = {}
    for n in of.NAMES:
        if n.startswith("W_"):
            w[n] = rng.normal(0, 0.4, (hm, hm))
        elif n == "b_out":
            w[n] = np.float64(0.3)
        else:
            w[n] = rng.normal(0, 0.5, hm)
    return w


def hand_model(b_out):
    w = {n: np.zeros((1, 1)) if n.startswith("W_") else np.zeros(1) for n in of.NAMES}
    w.update(w_mx=np.array([2.0]), W_mh=np.array([[3.0]]), w_hx=np.array([1.0]), W_hm=np.array([[1.0]]),
             w_out=np.array([1.0]), b_out=np.float64(b_out))
    return w


def test_normalised_two_step_forecasts_followed_by_hand():
    """tests/golden/forecaster_hand_cases.txt: a one-unit model on histories whose range is not 1, worked with
    a calculator: the min-max normalisation of the inputs (offset and range), the read-out taken back to
    token counts, a first forecast inside the history's range (same normalisation for the second step), one
    above it (the second step re-normalises over the extended history) and a flat history."""
    path = os.path.join(os.path.dirname(__file__), "golden", "forecaster_hand_cases.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert [r[0] for r in rows] == ["A", "B", "C"]
    for name, b_out, h0, h1, h2, want1, want2 in rows:
        y1, y2 = of.two_step_forecast(hand_model(float(b_out)), [float(h0), float(h1), float(h2)])
        assert abs(y1 - float(want1)) < 2e-9 * float(want1), name
        assert abs(y2 - float(want2)) < 2e-9 * float(want2), name


def test_normalisation_is_shift_and_scale_invariant():
    """The model only ever sees (v - min) / (max - min): histories a v + b (a > 0) give forecasts a y + b."""
    rng = np.random.default_rng(5)
    w = random_model(rng, 8)
    hist = rng.uniform(200, 3000, 10)
    y1, y2 = of.two_step_forecast(w, hist)
    z1, z2 = of.two_step_forecast(w, 7.5 * hist + 1e4)
    assert y1 > 0 and abs(z1 - (7.5 * y1 + 1e4)) < 1e-9 * z1 and abs(z2 - (7.5 * y2 + 1e4)) < 1e-9 * z2
    x, lo, span = of.normalise(hist)
    assert x.min() == 0.0 and x.max() == 1.0 and lo == hist.min() and span == hist.max() - hist.min()


def test_one_unit_two_steps_by_hand():
    """A single hidden unit with round weights, followed with a calculator."""
    w = {n: np.zeros((1, 1)) if n.startswith("W_") else np.zeros(1) for n in of.NAMES}
    w.update(w_mx=np.array([2.0]), W_mh=np.array([[3.0]]), w_hx=np.array([1.0]), W_hm=np.array([[1.0]]),
             w_out=np.array([1.0]), b_out=np.float64(0.0))
    # step 1, x = 0.5: m = (2*0.5)*(3*0) = 0; hh = 0.5; i = o = f = 1/2; c = tanh(0.5)/2; h = tanh(c)/2
    c1 = np.tanh(0.5) / 2
    h1 = np.tanh(c1) / 2
    # step 2, x = 1: m = 2 * 3 h1; hh = 1 + m; c = c1/2 + tanh(hh)/2; h = tanh(c)/2
    m2 = 6 * h1
    c2 = c1 / 2 + np.tanh(1 + m2) / 2
    h2 = np.tanh(c2) / 2
    h, c = of.mlstm_step(w, 0.5, np.zeros(1), np.zeros(1))
    assert abs(h[0] - h1) < 1e-15 and abs(c[0] - c1) < 1e-15
    h, c = of.mlstm_step(w, 1.0, h, c)
    assert abs(h[0] - h2) < 1e-15 and abs(c[0] - c2) < 1e-15
    # with tanh(0.5) = 0.462117, tanh(0.231059) = 0.227033, tanh(1.681098) = 0.933004, tanh(0.582031) = 0.524140
    assert abs(h[0] - 0.262070) < 2e-6


def test_reduces_to_a_plain_lstm_when_the_input_factor_is_one():
    """If w_mx x_t = 1 for the (constant) input, m_t = W_mh h_{t-1} and the cell is an LSTM whose
    recurrent matrices are W_*m W_mh: compared with torch's LSTMCell in fp64."""
    rng = np.random.default_rng(0)
    hm, x = 6, 0.8
    w = random_model(rng, hm)
    w["w_mx"] = np.full(hm, 1.0 / x)
    cell = torch.nn.LSTMCell(1, hm).double()
    with torch.no_grad():                                 # torch's gate order: input, forget, cell, output
        cell.weight_ih.copy_(torch.tensor(np.concatenate([w["w_ix"], w["w_fx"], w["w_hx"], w["w_ox"]])[:, None]))
        cell.weight_hh.copy_(torch.tensor(np.concatenate([w["W_im"] @ w["W_mh"], w["W_fm"] @ w["W_mh"],
                                                          w["W_hm"] @ w["W_mh"], w["W_om"] @ w["W_mh"]])))
        cell.bias_ih.copy_(torch.tensor(np.concatenate([w["b_i"], w["b_f"], w["b_h"], w["b_o"]])))
        cell.bias_hh.zero_()
    h, c = np.zeros(hm), np.zeros(hm)
    th, tc = torch.zeros(1, hm, dtype=torch.float64), torch.zeros(1, hm, dtype=torch.float64)
    for _ in range(7):
        h, c = of.mlstm_step(w, x, h, c)
        with torch.no_grad():
            th, tc = cell(torch.tensor([[x]], dtype=torch.float64), (th, tc))
    np.testing.assert_allclose(h, th.numpy()[0], rtol=0, atol=1e-14)
    np.testing.assert_allclose(c, tc.numpy()[0], rtol=0, atol=1e-14)


def test_second_step_is_the_model_on_the_extended_history():
    """Alg. 2: P' = P + {P_i}, then M(P').  While the first forecast stays inside the history's range the
    normalisation does not move and the second step is the recurrence carried on by one input."""
    rng = np.random.default_rng(1)
    w = random_model(rng, 16)
    w["w_out"] *= 0.2                                      # keeps the read-out inside (0, 1)
    hist = rng.uniform(200, 3000, 12)
    y1, y2 = of.two_step_forecast(w, hist)
    lo, hi = hist.min(), hist.max()
    assert lo < y1 < hi
    h, c = np.zeros(16), np.zeros(16)
    for v in np.append(hist, y1):
        h, c = of.mlstm_step(w, (v - lo) / (hi - lo), h, c)
    assert abs(y2 - (lo + (hi - lo) * (w["w_out"] @ h + w["b_out"]))) < 1e-9


def test_instance_count_formula():
    """N = max(P / mu_p, D / mu_d, (P + D) / mu_t).  A model with all weights zero and b_out = 1/2 forecasts the
    middle of its history's range: histories (0, 2 v) give v for the current and for the next window."""
    def half_model():
        w = {n: np.zeros((2, 2)) if n.startswith("W_") else np.zeros(2) for n in of.NAMES}
        w.update(b_out=np.float64(0.5))
        return w
    hist = lambda *v: np.array([[0.0, 2 * x] for x in v])
    out = of.forecast_services([half_model(), half_model()], [half_model(), half_model()],
                               hist(6000.0, 100.0), hist(900.0, 5000.0), mu_p=[2000.0, 2000.0], mu_d=[1000.0, 1000.0],
                               mu_t=[2500.0, 2500.0])
    assert out[0].tolist() == [6000.0, 100.0] and out[2].tolist() == [6000.0, 100.0]
    assert out[3].tolist() == [900.0, 5000.0]
    assert out[4].tolist() == [3.0, 5.0]                  # prefill-bound, then decode-bound
    out = of.forecast_services([half_model()], [half_model()], hist(1900.0), hist(900.0), [2000.0], [1000.0], [2500.0])
    assert abs(out[4][0] - 2800.0 / 2500.0) < 1e-15       # total-bound
