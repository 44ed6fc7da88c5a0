"""CPU oracle for the online phase of the service workload predictor (paper Sec. 3.2, Alg. 2): a
multiplicative LSTM per service and token kind forecasts the token count of the next time window from
the counts of the previous k windows, in two steps, and the counts are turned into a number of
instances.

TEST INFRASTRUCTURE ONLY: the plain definition the GPU library is checked against.  It shares no
code with the GPU path; only tests, the smoke check and the benchmark's CPU-baseline leg may call it.

The recurrence is the multiplicative LSTM of Krause et al. (2016), which the paper names: with scalar
input x_t (a window's token count divided by the model's `scale`), hidden state h and cell c,
    m_t = (w_mx x_t) * (W_mh h_{t-1})                      elementwise product
    hh  = w_hx x_t + W_hm m_t + b_h
    i_t = sigmoid(w_ix x_t + W_im m_t + b_i),  o_t, f_t likewise
    c_t = f_t * c_{t-1} + i_t * tanh(hh)
    h_t = tanh(c_t) * o_t
and the forecast after the last input is  y = scale * (w_out . h + b_out), not below 0.
Online phase (Alg. 2): step 1 forecasts the current window from the k past windows; the forecast is
appended to the history and step 2 forecasts the next window from the k + 1 values (the recurrence
simply goes on by one input).  With both kinds forecast, prompt tokens P and response tokens D,
    N = max(P / mu_p, D / mu_d, (P + D) / mu_t)
for the instance's profiled prefill, decode and total token capacities per window."""
from __future__ import annotations

import numpy as np

NAMES = ("w_mx", "W_mh", "w_hx", "W_hm", "b_h", "w_ix", "W_im", "b_i", "w_ox", "W_om", "b_o", "w_fx", "W_fm", "b_f",
         "w_out", "b_out", "scale")


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def mlstm_step(w, x, h, c):
    m = (w["w_mx"] * x) * (w["W_mh"] @ h)
    hh = w["w_hx"] * x + w["W_hm"] @ m + w["b_h"]
    i = sigmoid(w["w_ix"] * x + w["W_im"] @ m + w["b_i"])
    o = sigmoid(w["w_ox"] * x + w["W_om"] @ m + w["b_o"])
    f = sigmoid(w["w_fx"] * x + w["W_fm"] @ m + w["b_f"])
    c = f * c + i * np.tanh(hh)
    return np.tanh(c) * o, c


def readout(w, h):
    return max(0.0, float(w["scale"]) * (float(w["w_out"] @ h) + float(w["b_out"])))


def two_step_forecast(w, history):
    """(forecast of the current window, forecast of the next window) from the k past windows."""
    w = {k: np.asarray(v, np.float64) for k, v in w.items()}
    hm = w["W_mh"].shape[0]
    h, c = np.zeros(hm), np.zeros(hm)
    for v in np.asarray(history, np.float64):
        h, c = mlstm_step(w, v / float(w["scale"]), h, c)
    y1 = readout(w, h)
    h, c = mlstm_step(w, y1 / float(w["scale"]), h, c)
    return y1, readout(w, h)


def forecast_services(models_p, models_d, hist_p, hist_d, mu_p, mu_d, mu_t):
    """Per service s: (P_cur, D_cur, P_next, D_next, N_next) as float64 arrays."""
    S = len(models_p)
    out = np.zeros((5, S))
    for s in range(S):
        p1, p2 = two_step_forecast(models_p[s], hist_p[s])
        d1, d2 = two_step_forecast(models_d[s], hist_d[s])
        out[:, s] = (p1, d1, p2, d2, max(p2 / mu_p[s], d2 / mu_d[s], (p2 + d2) / mu_t[s]))
    return out
