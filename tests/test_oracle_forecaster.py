"""Pins for the CPU oracle of the service workload predictor's online phase (paper Sec. 3.2, Alg. 2)."""
import numpy as np
import torch

from oracle import forecaster as of


def random_model(rng, hm, scale=1000.0):
    w = {}
    for n in of.NAMES:
        if n.startswith("W_"):
            w[n] = rng.normal(0, 0.4, (hm, hm))
        elif n in ("b_out", "scale"):
            w[n] = np.float64(0.3 if n == "b_out" else scale)
        else:
            w[n] = rng.normal(0, 0.5, hm)
    return w


def test_one_unit_two_steps_by_hand():
    """A single hidden unit with round weights, followed with a calculator."""
    w = {n: np.zeros((1, 1)) if n.startswith("W_") else np.zeros(1) for n in of.NAMES}
    w.update(w_mx=np.array([2.0]), W_mh=np.array([[3.0]]), w_hx=np.array([1.0]), W_hm=np.array([[1.0]]),
             w_out=np.array([1.0]), b_out=np.float64(0.0), scale=np.float64(1.0))
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
    w = random_model(rng, hm, scale=1.0)
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
    rng = np.random.default_rng(1)
    w = random_model(rng, 16)
    hist = rng.uniform(200, 3000, 12)
    y1, y2 = of.two_step_forecast(w, hist)
    again, _ = of.two_step_forecast(w, np.append(hist, y1))      # Alg. 2: P' = P + {P_i}, then M(P')
    assert y1 >= 0 and abs(y2 - again) < 1e-9


def test_instance_count_formula():
    """N = max(P / mu_p, D / mu_d, (P + D) / mu_t) on forecasts fixed through the readout bias."""
    def const_model(value):
        w = {n: np.zeros((2, 2)) if n.startswith("W_") else np.zeros(2) for n in of.NAMES}
        w.update(b_out=np.float64(value), scale=np.float64(1.0))
        return w
    out = of.forecast_services([const_model(6000.0), const_model(100.0)], [const_model(900.0), const_model(5000.0)],
                               np.ones((2, 4)), np.ones((2, 4)), mu_p=[2000.0, 2000.0], mu_d=[1000.0, 1000.0],
                               mu_t=[2500.0, 2500.0])
    assert out[2].tolist() == [6000.0, 100.0] and out[3].tolist() == [900.0, 5000.0]
    assert out[4].tolist() == [3.0, 5.0]                  # prefill-bound, then decode-bound
    out = of.forecast_services([const_model(1900.0)], [const_model(900.0)], np.ones((1, 4)), np.ones((1, 4)),
                               [2000.0], [1000.0], [2500.0])
    assert abs(out[4][0] - 2800.0 / 2500.0) < 1e-15       # total-bound
